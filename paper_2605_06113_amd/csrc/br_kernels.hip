// gfx950 kernels of the BalanceRoute route step, except the sequential assignment
// (br_assign_kernel.h): state initialisation, decode step, horizon projection, and the
// F-score matrix with its stage-one reductions.
#include "br.h"
#include "br_device.h"
#include "br_launch.h"
#include "br_score_wave.h"

// ------------------------------------------------------------------ initialisation

__global__ void br_k_clear(BrParams p, int *pol) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t rows = (int64_t)p.N * p.G;
  if (tid < rows) {
    p.L[tid] = 0;
    p.n[tid] = 0;
  }
  if (tid < p.N) {
    p.qlen[tid] = 0;
    pol[2 * tid] = 0;
    pol[2 * tid + 1] = 0;
  }
}

// One wave per (cluster, worker): copy the caller's dense active list into the workspace
// layout and derive L_g = sum of kv (Sec. 2.2).
__global__ __launch_bounds__(256) void br_k_load_init(BrParams p, const int32_t *n_in, const int32_t *kv_in,
                                                     const int32_t *rem_in, const float *pred_in) {
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= (int64_t)p.N * p.G) return;  // whole wave leaves together
  const int lane = br_lane();
  int n_g = n_in[row];
  n_g = min(max(n_g, 0), p.B);
  int acc = 0;
  for (int j = lane; j < n_g; j += BR_WAVE) {
    const int kv = kv_in[row * p.B + j];
    p.kv[row * p.Bs + j] = kv;
    p.rem[row * p.Bs + j] = max(rem_in[row * p.B + j], 1);
    for (int q = 0; q < p.P; ++q) p.pred[(row * p.Bs + j) * p.P + q] = pred_in[(row * p.B + j) * p.P + q];
    acc += kv;
  }
  const int tot = br_wave_sum(acc);
  if (lane == 0) {
    p.L[row] = tot;
    p.n[row] = n_g;
  }
}

// ------------------------------------------------------------------ decode step
// Sec. 2.2: each active request advances one decode iteration per step: its KV length and
// the load of its worker grow by one token; after its last step it leaves and its whole KV
// footprint goes with it.  t steps are applied in closed form: a request with rem <= t
// leaves (net load change -kv), the others gain t tokens.  One wave owns one worker's dense
// list and compacts it in place, order preserved (writes never run ahead of reads).
template <int NC, int RW, bool PRED>
__global__ __launch_bounds__(256) void br_k_advance(BrParams p, int t) {
  // each wave owns RW consecutive worker lists, NC chunks of 256 slots each, four slots per lane;
  // everything it will touch is requested before the first result is needed, so that enough bytes
  // are in flight to cover the HBM latency, and the in-place compaction cannot overtake its own reads
  const int64_t row0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * RW;
  const int64_t rows = (int64_t)p.N * p.G;
  if (row0 >= rows) return;
  const int lane = br_lane();
  int n_g[RW];
  int4 kv[RW][NC], rem[RW][NC];
#pragma unroll
  for (int r = 0; r < RW; ++r) n_g[r] = row0 + r < rows ? p.n[row0 + r] : 0;
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int64_t base = (row0 + r) * p.Bs;
#pragma unroll
    for (int c = 0; c < NC; ++c) br_adv_load(p.kv + base, p.rem + base, c * 256 + 4 * lane, row0 + r < rows ? p.Bs : 0, kv[r][c], rem[r][c]);
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    if (row0 + r >= rows) break;
    const int64_t base = (row0 + r) * p.Bs;
    int kept = 0, gone = 0;  // uniform
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c * 256 < n_g[r]) {
        br_adv_apply<PRED>(p, t, c * 256 + 4 * lane, n_g[r], c * 256, kv[r][c], rem[r][c], p.kv + base, p.rem + base,
                           PRED ? p.pred + base * p.P : nullptr, kept, gone);
      }
    }
    if (lane == 0) {
      p.L[row0 + r] += kept * t - gone;  // survivors gain t tokens each
      p.n[row0 + r] = kept;
    }
  }
}
// The kernel is VALU-bound before it is HBM-bound (rocprofv3: ~500 vector instructions per wave with every
// loop written for 8 offsets and run-time widths), so the horizon bucket HB (4 or 8 offsets beyond h = 0), EXACT
// (H == HB: no per-offset conditions) and the kind of prediction row PK (0: a hazard per offset, 1: c_hat
// itself first in the row, 2: the pair (p_fin, mu_rem)) are compile-time.  c_hat of one active request (Appendix "Short-horizon prediction interface"): the survival sum
// of the hazards = E[min(r, H)] (eq. (two-stage)/(composite)) in sequential fp32, the p_fin gate and the floor
// of Appendix "Refresh logic", clip to [1, H]; or eq. (composite) on a supplied (p_fin, mu_rem) with the same gate;
// or the supplied / maintained value itself; all floored and clipped the same way.  A request counts kv + h at the offsets
// h <= floor(c_hat) (h is an integer, so that is (float)h <= c_hat; a NaN counts nowhere): per offset the kv
// part is summed in a register and over the wave, the count comes from a ballot.
template <int NC, int RW, int HB, bool EXACT, int PK>
__global__ __launch_bounds__(256) void br_k_project_rows(BrParams p) {
  constexpr bool HAZ = PK == 0;
  const int64_t row0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * RW;
  const int64_t rows = (int64_t)p.N * p.G;
  if (row0 >= rows) return;
  const int lane = br_lane();
  const int H1 = p.H + 1;
  const float Hf = (float)p.H;
  int n_g[RW], kv[RW][NC];
  float pr[RW][NC][HAZ ? HB : (PK == 2 ? 2 : 1)];
#pragma unroll
  for (int r = 0; r < RW; ++r) n_g[r] = row0 + r < rows ? p.n[row0 + r] : 0;
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int64_t base = (row0 + r) * p.Bs;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int j = c * BR_WAVE + lane;
      const bool used = j < n_g[r];
      kv[r][c] = used ? p.kv[base + j] : 0;
      const float *src = p.pred + (base + j) * p.P;
      if constexpr (PK == 2) {
        const float2 v = used ? *reinterpret_cast<const float2 *>(src) : make_float2(0.0f, 0.0f);
        pr[r][c][0] = v.x, pr[r][c][1] = v.y;
      } else if constexpr (!HAZ) {
        pr[r][c][0] = used ? src[0] : 0.0f;
      } else if constexpr (EXACT) {  // rows of HB floats: 16-byte loads
#pragma unroll
        for (int q = 0; q < HB; q += 4) {
          const float4 v = used ? *reinterpret_cast<const float4 *>(src + q) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
          pr[r][c][q] = v.x, pr[r][c][q + 1] = v.y, pr[r][c][q + 2] = v.z, pr[r][c][q + 3] = v.w;
        }
      } else {
#pragma unroll
        for (int q = 0; q < HB; ++q) pr[r][c][q] = (used && q < p.H) ? src[q] : 0.0f;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    if (row0 + r >= rows) break;
    int acc[HB + 1], cnt[HB + 1];
#pragma unroll
    for (int h = 0; h <= HB; ++h) acc[h] = 0, cnt[h] = 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int j = c * BR_WAVE + lane;
      float ch;
      if constexpr (HAZ) {
        float S = 1.0f;
        ch = 0.0f;
#pragma unroll
        for (int q = 0; q < HB; ++q) {
          if (EXACT || q < p.H) {
            ch = __fadd_rn(ch, S);
            S = __fmul_rn(S, __fsub_rn(1.0f, pr[r][c][q]));
          }
        }
        const float pfin = __fsub_rn(1.0f, S);
        if (p.gate > 0.0f && pfin < p.gate) ch = Hf;
      } else if constexpr (PK == 2) {
        const float pf = pr[r][c][0], mu = pr[r][c][1];
        ch = __fadd_rn(__fmul_rn(__fsub_rn(1.0f, pf), Hf), __fmul_rn(pf, mu));
        if (p.gate > 0.0f && pf < p.gate) ch = Hf;
      } else {
        ch = pr[r][c][0];
      }
      ch = ch < 1.0f ? 1.0f : ch;
      ch = ch > Hf ? Hf : ch;
      const int hm = (j < n_g[r] && ch >= 1.0f) ? (int)ch : -1;  // last offset the request counts at
#pragma unroll
      for (int h = 0; h <= HB; ++h) {
        if (EXACT || h <= p.H) {
          const bool in = h <= hm;
          acc[h] += in ? kv[r][c] : 0;
          cnt[h] += __builtin_popcountll(br_ballot(in));
        }
      }
    }
#pragma unroll
    for (int h = 0; h <= HB; ++h) {
      if (EXACT || h <= p.H) {
        const int v = br_wave_sum(acc[h]) + h * cnt[h];
        if (lane == 0) p.Lh[(row0 + r) * H1 + h] = v;
      }
    }
  }
}

// Horizons beyond BR_HP (Appendix "Short-horizon prediction interface", eq. (wprofile-new)): a request counts
// kv + h at the offsets h <= c_hat, so one histogram of floor(c_hat) per worker (count and kv sum, in LDS) and
// its suffix sums give L_g(k+h) = sum_{c >= h} kvsum[c] + h * sum_{c >= h} count[c] without a register per
// offset.  Integer sums, so the order of accumulation does not matter.  One block per cluster: each wave takes
// every fourth worker list and leaves its row in an LDS tile as well; then, with threads mapped to offsets,
// the envelope M_h = max_g L_g(k+h) and the margins, and with threads mapped to workers the horizon-min
// margin (what br_k_envelope does for short horizons in a launch of its own).
__global__ __launch_bounds__(256) void br_k_project_long(BrParams p) {
  extern __shared__ int lds[];
  const int wave = threadIdx.x >> 6, lane = br_lane(), tid = threadIdx.x;
  const int inst = blockIdx.x;
  const int G = p.G, H = p.H, H1 = H + 1, HS = BR_HS(H);
  int *tile = lds;                              // [G][HS] projections, then margins
  int *cnt = lds + G * HS + wave * 2 * HS;      // this wave's histogram: requests whose last offset is c
  int *kvs = cnt + HS;                          // ... and the sum of their kv
  const float Hf = (float)H;
  for (int g = wave; g < G; g += 4) {
    const int64_t row = (int64_t)inst * G + g;
    for (int h = lane; h < HS; h += BR_WAVE) cnt[h] = 0, kvs[h] = 0;
    br_wave_sync();
    const int n = min(max(p.n[row], 0), p.B);
    const int64_t base = row * p.Bs;
    int topc = 0, topk = 0;  // requests that reach the last offset (the gate's anchor: the common case)
    for (int j0 = 0; j0 < n; j0 += BR_WAVE) {
      const int j = j0 + lane;
      int kv = 0, hm = -1;
      if (j < n) {
        kv = p.kv[base + j];
        float c = p.pred[(base + j) * p.P];  // pred_mode 1 and 2 keep c_hat first
        if (p.pred_mode == 3) {              // the pair (p_fin, mu_rem): eq. (composite) and the gate
          const float pf = c, mu = p.pred[(base + j) * p.P + 1];
          c = __fadd_rn(__fmul_rn(__fsub_rn(1.0f, pf), Hf), __fmul_rn(pf, mu));
          if (p.gate > 0.0f && pf < p.gate) c = Hf;
        }
        c = c < 1.0f ? 1.0f : c;
        c = c > Hf ? Hf : c;
        if (c >= 0.0f) hm = min((int)c, H);  // offsets h with (float)h <= c_hat are 0..floor(c_hat); a NaN counts nowhere
      }
      const bool top = hm == H;
      topc += __builtin_popcountll(br_ballot(top));
      topk += br_wave_sum(top ? kv : 0);
      if (hm >= 0 && !top) {
        atomicAdd(&cnt[hm], 1);
        atomicAdd(&kvs[hm], kv);
      }
    }
    br_wave_sync();
    if (lane == 0) cnt[H] += topc, kvs[H] += topk;
    br_wave_sync();
    // suffix sums, four bins per trip: lane handles offsets lane, lane + 64, lane + 128
    int C[3] = {0, 0, 0}, K[3] = {0, 0, 0};
    for (int c4 = HS - 4; c4 >= 0; c4 -= 4) {
      const int4 cc = *reinterpret_cast<const int4 *>(cnt + c4);
      const int4 kk = *reinterpret_cast<const int4 *>(kvs + c4);
      const int cv[4] = {cc.x, cc.y, cc.z, cc.w}, kv4[4] = {kk.x, kk.y, kk.z, kk.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
          const bool in = c4 + e >= lane + u * BR_WAVE;
          C[u] += in ? cv[e] : 0;
          K[u] += in ? kv4[e] : 0;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const int h = lane + u * BR_WAVE;
      if (h < H1) {
        const int v = K[u] + h * C[u];
        p.Lh[row * H1 + h] = v;
        tile[g * HS + h] = v;
      }
    }
    br_wave_sync();  // the histogram is cleared again for this wave's next list
  }
  __syncthreads();
  if (tid < H1) {  // thread = offset
    int M = tile[tid];
    for (int g = 1; g < G; ++g) M = max(M, tile[g * HS + tid]);
    p.Mh[(int64_t)inst * H1 + tid] = M;
    for (int g = 0; g < G; ++g) {
      const int m = max(M - tile[g * HS + tid], 0);
      p.mh[((int64_t)inst * G + g) * H1 + tid] = m;
      tile[g * HS + tid] = m;
    }
  }
  __syncthreads();
  if (tid < G) {  // thread = worker
    int mn = INT32_MAX;
    for (int h = 0; h < H1; ++h) mn = min(mn, tile[tid * HS + h]);
    p.minm[(int64_t)inst * G + tid] = mn;
  }
}

// d = (1, gamma, ..., gamma^H) by repeated fp32 product (Sec. 4.1), zeros up to the padded length
__global__ void br_k_discounts(BrParams p, float gamma) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float *d = const_cast<float *>(p.dl);
  float dh = 1.0f;
  for (int h = 0; h < BR_HS(p.H); ++h) {
    if (h > 0) dh = __fmul_rn(dh, gamma);
    d[h] = h <= p.H ? dh : 0.0f;
  }
}

// Part 2: envelope M_h = max_g L_g(k+h), margins m_{g,h} = (M_h - L_g(k+h))_+ and min_h m_{g,h};
// one wave per cluster, lane g holds worker g.
__global__ __launch_bounds__(256) void br_k_envelope(BrParams p) {
  const int inst = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
  if (inst >= p.N) return;
  const int lane = br_lane();
  const bool act = lane < p.G;
  const int H1 = p.H + 1;
  const int64_t wrow = (int64_t)inst * p.G + lane;
  int mn = INT32_MAX;
  for (int h = 0; h < H1; ++h) {
    const int lh = act ? p.Lh[wrow * H1 + h] : BR_LOW;
    const int M = br_wave_max(lh);
    const int m = max(M - lh, 0);
    mn = min(mn, m);
    if (act) p.mh[wrow * H1 + h] = m;
    if (lane == 0) p.Mh[(int64_t)inst * H1 + h] = M;
  }
  if (act) p.minm[wrow] = mn;
}

// ------------------------------------------------------------------ F-score matrix + reductions
// Scores every (waiting request, worker) pair on the step-start snapshot: eq. (br0-Fscore) in
// int32 or eq. (brh-Fscore) in fp32.  Pass A maps lanes to requests (coalesced request-major
// reads, worker margins broadcast from LDS), reduces over workers in registers (best worker per
// request) and, if asked, stages the 64 x G tile in LDS so that the matrix leaves in full-width
// contiguous stores.  Pass B maps lanes to (request sub-slot, worker) and keeps a running best
// request per worker, combined across lanes and waves at the end.
// LONG (horizons beyond BR_HP): the margins keep BR_HS(H) entries per worker, the discounts sit in LDS next
// to them and a score loops over the offsets (br_scoreh_long), skipping the four-offset groups whose margins no
// request of the tile reaches.  want_tile == 2 (LONG, the cluster in one block, no matrix asked for): a score
// costs 3 (H + 1) operations here, so every pair is scored once: pass A stages its keys in the LDS tile and the
// running best request per worker is taken from the tile, tile by tile, instead of a second scoring pass.
template <bool BRH, bool LONG = false>
__global__ __launch_bounds__(512) void br_k_score(BrParams p, BrArr a, BrOut o, int want_tile) {
  extern __shared__ int lds[];
  const int G = p.G;
  const int HS = LONG ? BR_HS(p.H) : BR_HP + 1;  // margins per worker
  int *sm = lds;                         // [G][HS] margins
  float *sd = (float *)(sm + G * HS);    // LONG: [HS] discounts
  int *sL = sm + G * HS + (LONG ? HS : 0);  // [G]
  int *scap = sL + G;                    // [G]
  int *ss = scap + G;                    // [Q] prefill lengths of the waiting set
  int *cand = ss + p.Q;                  // [3][blockDim] candidates of pass B
  int *tiles = cand + 3 * blockDim.x;    // [waves][64][G+1] when the matrix is written out
  // a cluster may be spread over gridDim.y blocks: block `split` scores its share of the requests
  // against all workers (pass A) and all requests against its share of the workers (pass B), so no
  // result needs combining across blocks
  const int inst = blockIdx.x, split = blockIdx.y, nsplit = gridDim.y;
  const int tid = threadIdx.x, lane = br_lane(), wave = tid >> 6, nw = blockDim.x >> 6;

  const int q0 = min(max(p.qlen[inst], 0), p.Q);
  int cnt = a.count ? a.count[inst] : 0;
  cnt = min(max(cnt, 0), a.arr_cap);
  const int qn = q0 + min(cnt, p.Q - q0);

  if (tid < G) {
    sL[tid] = p.L[(int64_t)inst * G + tid];
    scap[tid] = p.B - p.n[(int64_t)inst * G + tid];
  }
  for (int e = tid; e < G * HS; e += blockDim.x) {
    const int g = e / HS, h = e - g * HS;
    const int m = (BRH && h <= p.H) ? p.mh[((int64_t)inst * G + g) * (p.H + 1) + h] : 0;
    sm[e] = LONG ? __float_as_int((float)m) : m;  // br_scoreh_long takes the margins as floats
  }
  if constexpr (LONG)
    for (int h = tid; h < HS; h += blockDim.x) sd[h] = p.dl[h];
  for (int i = tid; i < qn; i += blockDim.x) {
    int s = i < q0 ? p.qs[(int64_t)inst * p.Q + i] : a.s[(int64_t)inst * a.arr_cap + (i - q0)];
    ss[i] = min(max(s, 1), BR_MAX_S_DEV);
  }
  __syncthreads();
  if (!BRH) {  // M(k) = max_g L_g, m_g = M - L_g
    if (tid < G) {
      int M = sL[0];
      for (int g = 1; g < G; ++g) M = max(M, sL[g]);
      sm[tid * HS] = M - sL[tid];
    }
    __syncthreads();
  }

  // running best request per worker when pass B reads the staged keys (want_tile == 2): lane = (sub-slot, worker)
  const bool once = LONG && want_tile == 2 && o.best_i;
  int Gp1 = 1;
  while (Gp1 < G) Gp1 <<= 1;
  const int nsub1 = BR_WAVE / Gp1, sub1 = lane / Gp1, gl1 = lane - sub1 * Gp1;
  const bool act1 = gl1 < G;
  const bool free1 = act1 && scap[act1 ? gl1 : 0] > 0;
  const int Lg1 = act1 ? sL[gl1] : 0;
  int bk1 = BR_KEY_NONE, bs1 = 0, bi1 = -1;

  // pass A: one request per lane, loop over workers
  int *tile = tiles + wave * (BR_WAVE * (G + 1));
  for (int t0 = (split * nw + wave) * BR_WAVE; t0 < qn; t0 += nsplit * nw * BR_WAVE) {
    const int i = t0 + lane;
    const bool valid = i < qn;
    const int s = valid ? ss[i] : 1;
    int bk = BR_KEY_NONE, bg = -1;
    int tile_top[1] = {0};
    if constexpr (LONG) tile_top[0] = br_wave_max(valid ? s : 0);  // the longest request of the tile
    for (int g = 0; g < G; ++g) {
      int key;
      if constexpr (LONG) {
        const int dv[1] = {s};
        float Fv[1];
        br_scoreh_long_sel<1>(p.aD, p.beta, (const float *)(sm + g * HS), sd, HS, lane, tile_top, dv, Fv);
        key = br_ord(Fv[0]);
      } else {
        int m[BR_HP + 1];
#pragma unroll
        for (int h = 0; h <= BR_HP; ++h) m[h] = (BRH || h == 0) ? sm[g * (BR_HP + 1) + h] : 0;
        key = br_score_key<BRH>(p, m, s);
      }
      if (want_tile) tile[lane * (G + 1) + g] = key;
      const bool ok = scap[g] > 0 && (p.W <= 0 || sL[g] + s <= p.W);
      if (ok && key > bk) {
        bk = key;
        bg = g;
      }
    }
    if (valid && o.best_g) o.best_g[(int64_t)inst * p.Q + i] = bg;
    if (once) {  // this tile's keys against the running best of every worker (ascending requests within a lane)
      br_wave_sync();
      const int rows = min(BR_WAVE, qn - t0);
      for (int r = sub1; r < rows; r += nsub1) {
        const int sr = ss[t0 + r];
        const int key = tile[r * (G + 1) + (act1 ? gl1 : 0)];
        const bool ok = free1 && (p.W <= 0 || Lg1 + sr <= p.W);
        if (ok && (key > bk1 || (key == bk1 && sr > bs1))) {
          bk1 = key;
          bs1 = sr;
          bi1 = t0 + r;
        }
      }
      br_wave_sync();  // the tile is rewritten by the wave's next trip
    }
    if (want_tile == 1) {
      const int rows = min(BR_WAVE, qn - t0);
      int *Fi = (int *)o.F + ((int64_t)inst * p.Q + t0) * G;
      for (int e = lane; e < rows * G; e += BR_WAVE) {
        const int r = e / G, g = e - r * G;
        const int key = tile[r * (G + 1) + g];
        Fi[e] = BRH ? __float_as_int(br_unord(key)) : key;
      }
    }
  }
  if (o.best_g && split == 0)
    for (int i = qn + tid; i < p.Q; i += blockDim.x) o.best_g[(int64_t)inst * p.Q + i] = -1;

  // pass B: lane = (sub-slot, worker of this block's share); running best request per worker
  if (o.best_i) {
    const int Gs = (G + nsplit - 1) / nsplit, gbase = split * Gs;  // workers [gbase, gbase + Gs)
    int Gp = 1;
    while (Gp < Gs) Gp <<= 1;
    const int nsub = BR_WAVE / Gp;
    const int sub = lane / Gp, gl = lane - sub * Gp, g = gbase + gl;
    const bool act = gl < Gs && g < G;
    int m[BR_HP + 1];
#pragma unroll
    for (int h = 0; h <= BR_HP; ++h) m[h] = (!LONG && act && (BRH || h == 0)) ? sm[g * (BR_HP + 1) + h] : 0;
    const int Lg = act ? sL[g] : 0;
    const bool free_slot = act && scap[g] > 0;
    int bk = BR_KEY_NONE, bs = 0, bi = -1;
    if (once) bk = bk1, bs = bs1, bi = bi1;  // (one block holds the cluster: the lane layout is the one above)
    for (int i = wave * nsub + sub; i < qn && !once; i += nw * nsub) {
      const int s = ss[i];
      int key;
      if constexpr (LONG) {  // lanes hold different workers: each reads its own row of margins
        const int dv[1] = {s};
        float Fv[1];
        br_scoreh_long<1>(p.aD, p.beta, (const float *)(sm + (act ? g : 0) * HS), sd, HS, dv, Fv);
        key = br_ord(Fv[0]);
      } else {
        key = br_score_key<BRH>(p, m, s);
      }
      const bool ok = free_slot && (p.W <= 0 || Lg + s <= p.W);
      if (ok && (key > bk || (key == bk && s > bs))) {
        bk = key;
        bs = s;
        bi = i;
      }
    }
    cand[tid] = bk;
    cand[blockDim.x + tid] = bs;
    cand[2 * blockDim.x + tid] = bi;
    __syncthreads();
    if (tid < Gs && gbase + tid < G) {
      bk = BR_KEY_NONE, bs = 0, bi = -1;
      for (int w = 0; w < nw; ++w)
        for (int sb = 0; sb < nsub; ++sb) {
          const int c = w * BR_WAVE + sb * Gp + tid;
          const int k = cand[c], s = cand[blockDim.x + c], i = cand[2 * blockDim.x + c];
          if (i < 0) continue;
          if (bi < 0 || k > bk || (k == bk && (s > bs || (s == bs && i < bi)))) {
            bk = k;
            bs = s;
            bi = i;
          }
        }
      o.best_i[(int64_t)inst * G + gbase + tid] = bi;
    }
  }
}

// K2 with the matrix materialised: every (waiting request, worker) score of the step-start snapshot written to
// HBM, request-major (F[inst][i][g]), and nothing else: the reductions run as their own launch without it.
// An HBM-write stream: one block per cluster; margins and prefill lengths are staged in LDS once, then every
// thread computes the four scores of one 16-byte store straight in the output's layout (element e of the
// cluster's rows is request e / G, worker e % G, by a multiply-high with the rounded-up reciprocal of G, exact for
// e < 2^17), so the matrix leaves in full-width contiguous stores and no tile is staged.  Rows at or beyond the
// queue length are left untouched.
template <bool BRH, bool LONG>
__global__ __launch_bounds__(256) void br_k_score_matrix(BrParams p, BrArr a, BrOut o, unsigned recip_g) {
  extern __shared__ int lds[];
  const int G = p.G;
  const int HS = LONG ? BR_HS(p.H) : BR_HP + 1;
  int *sm = lds;                                   // [G][HS] margins (LONG: as floats)
  float *sd = (float *)(sm + G * HS);              // LONG: [HS + 4] discounts
  int *ss = sm + G * HS + (LONG ? HS + 4 : 0);     // [Q] prefill lengths
  int *sL = ss + p.Q;                              // [G] loads (BR-0)
  const int inst = blockIdx.x, tid = threadIdx.x;
  const int q0 = min(max(p.qlen[inst], 0), p.Q);
  int cnt = a.count ? a.count[inst] : 0;
  cnt = min(max(cnt, 0), a.arr_cap);
  const int qn = q0 + min(cnt, p.Q - q0);
  if (!BRH && tid < G) sL[tid] = p.L[(int64_t)inst * G + tid];
  for (int e = tid; e < G * HS; e += blockDim.x) {
    const int g = e / HS, h = e - g * HS;
    const int m = (BRH && h <= p.H) ? p.mh[((int64_t)inst * G + g) * (p.H + 1) + h] : 0;
    sm[e] = LONG ? __float_as_int((float)m) : m;
  }
  if constexpr (LONG)
    for (int h = tid; h < HS + 4; h += blockDim.x) sd[h] = h < HS ? p.dl[h] : 0.0f;
  for (int i = tid; i < qn; i += blockDim.x) {
    const int s = i < q0 ? p.qs[(int64_t)inst * p.Q + i] : a.s[(int64_t)inst * a.arr_cap + (i - q0)];
    ss[i] = min(max(s, 1), BR_MAX_S_DEV);
  }
  __syncthreads();
  if (!BRH) {  // M(k) = max_g L_g, m_g = M - L_g
    if (tid < G) {
      int M = sL[0];
      for (int g = 1; g < G; ++g) M = max(M, sL[g]);
      sm[tid * HS] = M - sL[tid];
    }
    __syncthreads();
  }
  int *Fi = (int *)o.F + (int64_t)inst * p.Q * G;   // 16-byte aligned: Q * G * 4 bytes per cluster with Q * G % 4 == 0 or a scalar tail
  const int total = qn * G;
  auto score_at = [&](int e) -> int {
    const int i = G == 1 ? e : (int)__umulhi((unsigned)e, recip_g), g = e - i * G;
    int key;
    if constexpr (LONG) {
      const int dv[1] = {ss[i]};
      float Fv[1];
      br_scoreh_long<1>(p.aD, p.beta, (const float *)(sm + g * HS), sd, HS, dv, Fv);
      return __float_as_int(Fv[0]);
    } else {
      int m[BR_HP + 1];
#pragma unroll
      for (int h = 0; h <= BR_HP; ++h) m[h] = (BRH || h == 0) ? sm[g * (BR_HP + 1) + h] : 0;
      key = br_score_key<BRH>(p, m, ss[i]);
      return BRH ? __float_as_int(br_unord(key)) : key;
    }
  };
  const bool vec = (((int64_t)inst * p.Q * G) & 3) == 0;   // the cluster's rows start on a 16-byte boundary
  if (vec) {
    for (int e = 4 * tid; e < total; e += 4 * blockDim.x) {
      if (e + 3 < total) {
        *reinterpret_cast<int4 *>(Fi + e) = make_int4(score_at(e), score_at(e + 1), score_at(e + 2), score_at(e + 3));
      } else {
        for (int k = e; k < total; ++k) Fi[k] = score_at(k);
      }
    }
  } else {
    for (int e = tid; e < total; e += blockDim.x) Fi[e] = score_at(e);
  }
}

// K2 + K3 for a few clusters with long queues (single-instance serving): the block-per-cluster kernel above
// leaves most of the chip idle and its two passes score every pair twice.  Here one wave takes a tile of 64
// requests against a quarter of the workers (grid: tiles x 4 worker groups x clusters), scores each pair
// once, keeps the best worker of its group per request in registers and finds the best request of its tile per
// worker by three wave reductions (score, then length, then arrival position: the tie rule of br_k_score).
// The partial results go to a scratch area of the workspace; br_k_score_combine folds them (groups in
// ascending worker order, tiles in ascending request order, so ties resolve as in the one-block kernel).
// Scratch per cluster: pg_key, pg_g [WGN][Q]; pi_key, pi_s, pi_i [T][G].
#define BR_TILE_WORKERS 16  // most workers in a group (64 workers in 4 groups)
#define BR_TILE_GROUPS 4
__host__ __device__ inline size_t br_score_scratch_words(int Q, int G) {
  const size_t T = (size_t)(Q + BR_WAVE - 1) / BR_WAVE;
  return 2 * BR_TILE_GROUPS * (size_t)Q + 3 * T * (size_t)G;
}

template <bool BRH, bool LONG>
__global__ __launch_bounds__(64) void br_k_score_tiles(BrParams p, BrArr a, int *partials, int wpg) {
  extern __shared__ int lds[];
  const int tile = blockIdx.x, wg = blockIdx.y, inst = blockIdx.z;
  const int T = gridDim.x, WGN = gridDim.y;
  const int lane = br_lane(), G = p.G;
  const int g0 = wg * wpg, gn = min(wpg, G - g0);  // wpg <= BR_TILE_WORKERS workers per group
  const int HS = LONG ? BR_HS(p.H) : BR_HP + 1;
  int *sm = lds;                                      // [16][HS] margins of the group's workers (LONG: as floats)
  float *sd = (float *)(sm + BR_TILE_WORKERS * HS);   // LONG: [HS] discounts (+ 4 words read ahead)
  int *sL = sm + BR_TILE_WORKERS * HS + (LONG ? HS + 4 : 0);  // [16] loads, then [16] free slots
  int *scap = sL + BR_TILE_WORKERS;
  int *sc = partials + (size_t)inst * br_score_scratch_words(p.Q, G);
  int *pg_key = sc, *pg_g = sc + (size_t)WGN * p.Q;
  int *pi_key = sc + 2 * (size_t)WGN * p.Q, *pi_s = pi_key + (size_t)T * G, *pi_i = pi_s + (size_t)T * G;

  const int q0 = min(max(p.qlen[inst], 0), p.Q);
  int cnt = a.count ? a.count[inst] : 0;
  cnt = min(max(cnt, 0), a.arr_cap);
  const int qn = q0 + min(cnt, p.Q - q0);

  // worker state of the group; BR-0 margins need the envelope over all workers
  const int Lall = lane < G ? p.L[(int64_t)inst * G + lane] : BR_LOW;
  const int M = br_wave_max(Lall);
  if (lane < gn) {
    sL[lane] = p.L[(int64_t)inst * G + g0 + lane];
    scap[lane] = p.B - p.n[(int64_t)inst * G + g0 + lane];
  }
  for (int e = lane; e < gn * HS; e += BR_WAVE) {
    const int gl = e / HS, h = e - gl * HS;
    int m = 0;
    if (BRH) {
      if (h <= p.H) m = p.mh[((int64_t)inst * G + g0 + gl) * (p.H + 1) + h];
    } else if (h == 0) {
      m = M - p.L[(int64_t)inst * G + g0 + gl];
    }
    sm[e] = LONG ? __float_as_int((float)m) : m;
  }
  if constexpr (LONG)
    for (int h = lane; h < HS + 4; h += BR_WAVE) sd[h] = h < HS ? p.dl[h] : 0.0f;
  br_wave_sync();

  const int i = tile * BR_WAVE + lane;
  const bool valid = i < qn;
  int s = 1;
  if (valid) s = i < q0 ? p.qs[(int64_t)inst * p.Q + i] : a.s[(int64_t)inst * a.arr_cap + (i - q0)];
  s = min(max(s, 1), BR_MAX_S_DEV);
  int bk = BR_KEY_NONE, bg = -1;
  for (int gl = 0; gl < gn; ++gl) {
    int key;
    if constexpr (LONG) {
      const int dv[1] = {s};
      float Fv[1];
      br_scoreh_long<1>(p.aD, p.beta, (const float *)(sm + gl * HS), sd, HS, dv, Fv);
      key = br_ord(Fv[0]);
    } else {
      int m[BR_HP + 1];
#pragma unroll
      for (int h = 0; h <= BR_HP; ++h) m[h] = (BRH || h == 0) ? sm[gl * HS + h] : 0;
      key = br_score_key<BRH>(p, m, s);
    }
    const bool ok = valid && scap[gl] > 0 && (p.W <= 0 || sL[gl] + s <= p.W);
    if (ok && key > bk) {  // workers in ascending order: the first best stays
      bk = key;
      bg = g0 + gl;
    }
    // best request of this tile for worker g: score, then the longer request, then the earlier arrival
    const int kk = ok ? key : BR_KEY_NONE;
    const int km = br_wave_max(kk);
    int sbest = 0, ibest = -1;
    if (km != BR_KEY_NONE) {
      sbest = br_wave_max(kk == km ? s : -1);
      ibest = br_wave_min((kk == km && s == sbest) ? i : INT32_MAX);
    }
    if (lane == 0) {
      const size_t at = (size_t)tile * G + g0 + gl;
      pi_key[at] = km, pi_s[at] = sbest, pi_i[at] = ibest;
    }
  }
  if (i < p.Q) {
    pg_key[(size_t)wg * p.Q + i] = bk;
    pg_g[(size_t)wg * p.Q + i] = bg;
  }
}

// Blocks [0, QB) fold the per-group best workers of 256 requests each; the others take four workers each, one
// wave per worker with lanes mapped to tiles (at most 32), and fold the per-tile best requests by the same three
// reductions.  All partial results are requested at once: nothing here waits on a load more than once.
__global__ __launch_bounds__(256) void br_k_score_combine(BrParams p, BrOut o, const int *partials, int T, int WGN, int QB) {
  const int inst = blockIdx.y, tid = threadIdx.x, G = p.G;
  const int *sc = partials + (size_t)inst * br_score_scratch_words(p.Q, G);
  const int *pg_key = sc, *pg_g = sc + (size_t)WGN * p.Q;
  const int *pi_key = sc + 2 * (size_t)WGN * p.Q, *pi_s = pi_key + (size_t)T * G, *pi_i = pi_s + (size_t)T * G;
  if ((int)blockIdx.x < QB) {
    const int i = blockIdx.x * 256 + tid;
    if (!o.best_g || i >= p.Q) return;
    int k[4], gg[4];
#pragma unroll
    for (int wg = 0; wg < 4; ++wg) {
      k[wg] = wg < WGN ? pg_key[(size_t)wg * p.Q + i] : BR_KEY_NONE;
      gg[wg] = wg < WGN ? pg_g[(size_t)wg * p.Q + i] : -1;
    }
    int bk = BR_KEY_NONE, bg = -1;
#pragma unroll
    for (int wg = 0; wg < 4; ++wg)
      if (k[wg] > bk) bk = k[wg], bg = gg[wg];
    o.best_g[(int64_t)inst * p.Q + i] = bg;
  } else {
    const int g = ((int)blockIdx.x - QB) * 4 + (tid >> 6), lane = br_lane();
    if (!o.best_i || g >= G) return;  // whole waves leave
    const bool in = lane < T;
    const int i = in ? pi_i[(size_t)lane * G + g] : -1;
    const int k = in ? pi_key[(size_t)lane * G + g] : BR_KEY_NONE;
    const int s = in ? pi_s[(size_t)lane * G + g] : 0;
    const int kk = i >= 0 ? k : BR_KEY_NONE;
    const int km = br_wave_max(kk);
    int bi = -1;
    if (km != BR_KEY_NONE) {
      const int sbest = br_wave_max(kk == km ? s : -1);
      bi = br_wave_min((kk == km && s == sbest) ? i : INT32_MAX);
    }
    if (lane == 0) o.best_i[(int64_t)inst * G + g] = bi;
  }
}

// K2 + K3, one wave per cluster (br_score_wave.h)
template <int E, bool BRH>
__global__ __launch_bounds__(256) void br_k_score_wave(BrParams p, BrArr a, BrOut o) {
  const int inst = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
  if (inst >= p.N) return;
  const int lane = br_lane();
  BrScoreIn<E, BRH> in;
  br_score_wave_load<E, BRH>(p, a, inst, lane, in);
  br_score_wave_run<E, BRH>(p, o, inst, lane, in);
}

// ------------------------------------------------------------------ launchers

void br_launch_clear(const BrParams &p, int *pol, hipStream_t st) {
  const int64_t n = (int64_t)p.N * p.G;
  hipLaunchKernelGGL(br_k_clear, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, pol);
}

void br_launch_load_init(const BrParams &p, const int32_t *n, const int32_t *kv, const int32_t *rem, const float *pred,
                         hipStream_t st) {
  const int64_t rows = (int64_t)p.N * p.G;
  hipLaunchKernelGGL(br_k_load_init, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, p, n, kv, rem, pred);
}

template <int NC, int RW>
static void launch_advance(const BrParams &p, int t, hipStream_t st) {
  constexpr int RWP = NC == 1 ? 2 : 1;  // lists that carry prediction rows: at most four chunks per wave (code size)
  if (p.P) {
    const int64_t waves = ((int64_t)p.N * p.G + RWP - 1) / RWP;
    hipLaunchKernelGGL((br_k_advance<NC, RWP, true>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, p, t);
  } else {
    const int64_t waves = ((int64_t)p.N * p.G + RW - 1) / RW;
    hipLaunchKernelGGL((br_k_advance<NC, RW, false>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, p, t);
  }
}

void br_launch_advance(const BrParams &p, int t, hipStream_t st) {
  if (p.Bs <= 256)
    launch_advance<1, 2>(p, t, st);
  else if (p.Bs <= 512)
    launch_advance<2, 4>(p, t, st);
  else
    launch_advance<4, 2>(p, t, st);
}

template <int NC, int RW, int HB, bool EXACT>
static void launch_project_rows_h(const BrParams &p, hipStream_t st) {
  const int64_t waves = ((int64_t)p.N * p.G + RW - 1) / RW;
  const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  if (p.pred_mode == 0)
    hipLaunchKernelGGL((br_k_project_rows<NC, RW, HB, EXACT, 0>), grid, block, 0, st, p);
  else if (p.pred_mode == 3)
    hipLaunchKernelGGL((br_k_project_rows<NC, RW, HB, EXACT, 2>), grid, block, 0, st, p);
  else
    hipLaunchKernelGGL((br_k_project_rows<NC, RW, HB, EXACT, 1>), grid, block, 0, st, p);
}

template <int NC, int RW>
static void launch_project_rows(const BrParams &p, hipStream_t st) {
  if (p.H == 4)
    launch_project_rows_h<NC, RW, 4, true>(p, st);
  else if (p.H == 8)
    launch_project_rows_h<NC, RW, 8, true>(p, st);
  else if (p.H < 4)
    launch_project_rows_h<NC, RW, 4, false>(p, st);
  else
    launch_project_rows_h<NC, RW, 8, false>(p, st);
}

void br_launch_discounts(const BrParams &p, float gamma, hipStream_t st) {
  hipLaunchKernelGGL(br_k_discounts, dim3(1), dim3(64), 0, st, p, gamma);
}

void br_launch_project(const BrParams &p, hipStream_t st) {
  if (p.H > BR_HP) {  // projection, envelope and margins in one launch
    const size_t lds = ((size_t)p.G + 8) * BR_HS(p.H) * sizeof(int);
    hipLaunchKernelGGL(br_k_project_long, dim3((unsigned)p.N), dim3(256), lds, st, p);
    return;
  }
  if (p.B <= 64)
    launch_project_rows<1, 4>(p, st);
  else if (p.B <= 128)
    launch_project_rows<2, 2>(p, st);
  else if (p.B <= 192)
    launch_project_rows<3, 2>(p, st);
  else if (p.B <= 256)
    launch_project_rows<4, 2>(p, st);
  else if (p.B <= 512)
    launch_project_rows<8, 1>(p, st);
  else
    launch_project_rows<16, 1>(p, st);
  hipLaunchKernelGGL(br_k_envelope, dim3((unsigned)((p.N + 3) / 4)), dim3(256), 0, st, p);
}

size_t br_score_scratch_bytes(int N, int Q, int G) {
  return N <= BR_SCORE_TILES_MAX_N ? (size_t)N * br_score_scratch_words(Q, G) * sizeof(int) : 0;
}

// The same partial results for callers that cannot allocate (br_route_step_static): a fixed device array in
// place of the workspace area, large enough for the most the tiled path ever needs (BR_SCORE_TILES_MAX_N
// clusters with the longest queue and the most workers: 1.4 MB).  Every GPU holds its own copy until the
// process ends.  Host code never uses the array by name: its address on a device comes from
// hipGetSymbolAddress, once per device, and the kernels get that pointer as an argument like any other buffer.
// Both kernels write every entry they later read, so nothing has to be cleared between calls; calls that
// overlap on one GPU (two streams) would race on it.
#define BR_STATIC_SCRATCH_WORDS (BR_SCORE_TILES_MAX_N * (2 * BR_TILE_GROUPS * 2048 + 3 * 32 * 64))
static __device__ __align__(256) int scratch[BR_STATIC_SCRATCH_WORDS];
static_assert(BR_STATIC_SCRATCH_WORDS * sizeof(int) == BR_STATIC_SCRATCH_BYTES && BR_SCORE_TILES_MAX_N == BR_STATIC_MAX_INST &&
                  BR_MAX_WAIT == 2048 && BR_MAX_G == 64,
              "the fixed scratch array covers the largest tiled score launch");

#define BR_MAX_DEVICES 64
static int *g_static_scratch[BR_MAX_DEVICES];  // device address of `scratch` per device, once resolved

size_t br_static_scratch_bytes() { return (size_t)BR_STATIC_SCRATCH_WORDS * sizeof(int); }

// Address of this library's static scratch array on the CURRENT device (resolved once per device).
hipError_t br_static_scratch_resolve(int **out) {
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= BR_MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_static_scratch[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_static_scratch[dev] = (int *)ptr;
  }
  *out = g_static_scratch[dev];
  return hipSuccess;
}

static void br_launch_reductions(const BrParams &p, const BrArr &a, const BrOut &o, int *partials, hipStream_t st);

void br_launch_score(const BrParams &p, const BrArr &a, const BrOut &o, int *partials, hipStream_t st) {
  if (o.F) {  // the matrix as a stream of its own; the reductions, if asked for, by whichever kernel serves the shape
    const bool longh = p.H > BR_HP;
    const size_t HS = longh ? BR_HS(p.H) : BR_HP + 1;
    const size_t lds = ((size_t)p.G * HS + (longh ? HS + 4 : 0) + (size_t)p.Q + (size_t)p.G) * sizeof(int);
    const unsigned recip = (unsigned)((0x100000000ull + (unsigned)p.G - 1u) / (unsigned)p.G);  // ceil(2^32 / G)
    if (longh)
      hipLaunchKernelGGL((br_k_score_matrix<true, true>), dim3((unsigned)p.N), dim3(256), lds, st, p, a, o, recip);
    else if (p.H > 0)
      hipLaunchKernelGGL((br_k_score_matrix<true, false>), dim3((unsigned)p.N), dim3(256), lds, st, p, a, o, recip);
    else
      hipLaunchKernelGGL((br_k_score_matrix<false, false>), dim3((unsigned)p.N), dim3(256), lds, st, p, a, o, recip);
    if (!o.best_g && !o.best_i) return;
    BrOut o2 = o;
    o2.F = nullptr;
    br_launch_reductions(p, a, o2, partials, st);
    return;
  }
  br_launch_reductions(p, a, o, partials, st);
}

static void br_launch_reductions(const BrParams &p, const BrArr &a, const BrOut &o, int *partials, hipStream_t st) {
  int waves = (p.Q + 63) / 64;  // one wave per tile of 64 requests, at most 8 waves
  waves = waves < 1 ? 1 : (waves > 8 ? 8 : waves);
  const int want_tile = o.F != nullptr;
  const bool longh = p.H > BR_HP;
  {  // few clusters, long queues, no matrix: a wave per (tile of requests, group of workers), then a combine
    const int T = (p.Q + BR_WAVE - 1) / BR_WAVE;
    const int wpg = (p.G + BR_TILE_GROUPS - 1) / BR_TILE_GROUPS, WGN = (p.G + wpg - 1) / wpg;  // at most 4 groups
    if (partials && !want_tile && p.N <= BR_SCORE_TILES_MAX_N && T * WGN >= 8) {
      const dim3 grid((unsigned)T, (unsigned)WGN, (unsigned)p.N), block(BR_WAVE);
      const int HS = longh ? BR_HS(p.H) : BR_HP + 1;
      const size_t lds = ((size_t)BR_TILE_WORKERS * HS + (longh ? HS + 4 : 0) + 2 * BR_TILE_WORKERS) * sizeof(int);
      if (longh)
        hipLaunchKernelGGL((br_k_score_tiles<true, true>), grid, block, lds, st, p, a, partials, wpg);
      else if (p.H > 0)
        hipLaunchKernelGGL((br_k_score_tiles<true, false>), grid, block, lds, st, p, a, partials, wpg);
      else
        hipLaunchKernelGGL((br_k_score_tiles<false, false>), grid, block, lds, st, p, a, partials, wpg);
      const int QB = (p.Q + 255) / 256;
      hipLaunchKernelGGL(br_k_score_combine, dim3((unsigned)(QB + (p.G + 3) / 4), (unsigned)p.N), dim3(256), 0, st, p, o,
                         (const int *)partials, T, WGN, QB);
      return;
    }
  }
  if (!longh && !want_tile && p.Q <= 512 && p.N >= BR_SCORE_WAVE_MIN_N) {  // many small clusters: one wave each
    const dim3 grid((unsigned)((p.N + 3) / 4)), block(256);
    if (p.H > 0) {
      if (p.Q <= 256)
        hipLaunchKernelGGL((br_k_score_wave<4, true>), grid, block, 0, st, p, a, o);
      else
        hipLaunchKernelGGL((br_k_score_wave<8, true>), grid, block, 0, st, p, a, o);
    } else {
      if (p.Q <= 256)
        hipLaunchKernelGGL((br_k_score_wave<4, false>), grid, block, 0, st, p, a, o);
      else
        hipLaunchKernelGGL((br_k_score_wave<8, false>), grid, block, 0, st, p, a, o);
    }
    return;
  }
  auto lds_words = [&](int w, bool tile) {
    const size_t HS = longh ? BR_HS(p.H) : BR_HP + 1;
    size_t words = (size_t)p.G * HS + (longh ? HS : 0) + 2 * (size_t)p.G + (size_t)p.Q + 3 * 64 * (size_t)w;
    if (tile) words += (size_t)w * 64 * (size_t)(p.G + 1);
    return words;
  };
  while (waves > 1 && lds_words(waves, want_tile) * 4 > 60 * 1024) --waves;  // stay within the default 64 KiB of LDS per block
  size_t lds = lds_words(waves, want_tile) * 4;
  // few clusters: spread each over several blocks (at most 8, at most one per worker) to fill more CUs
  int nsplit = 1;
  while (nsplit < 8 && nsplit * 2 <= p.G && (int64_t)p.N * nsplit * 2 <= 512 && p.Q > 64 * waves * nsplit) nsplit *= 2;
  const dim3 grid((unsigned)p.N, (unsigned)nsplit);
  // long horizons, the cluster in one block, room for the staged keys: every pair is scored once
  int mode = want_tile;
  if (longh && !want_tile && nsplit == 1 && o.best_i && lds_words(waves, true) * 4 <= 60 * 1024) {
    mode = 2;
    lds = lds_words(waves, true) * 4;
  }
  if (longh)
    hipLaunchKernelGGL((br_k_score<true, true>), grid, dim3(64 * waves), lds, st, p, a, o, mode);
  else if (p.H > 0)
    hipLaunchKernelGGL(br_k_score<true>, grid, dim3(64 * waves), lds, st, p, a, o, want_tile);
  else
    hipLaunchKernelGGL(br_k_score<false>, grid, dim3(64 * waves), lds, st, p, a, o, want_tile);
}
