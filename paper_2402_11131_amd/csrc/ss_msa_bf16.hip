// a2, bf16 path: multi-stream attention (Eq. 1 / Eq. 2) on the gfx950 matrix cores.
//
// Work split.  A workgroup (4 wavefronts, one per SIMD) owns one (sequence, KV
// head, split of the cached tokens, chunk of <= 80 folded query rows).  The
// query heads of a GQA group are folded into the row dimension, so K and V are
// read once per KV head.  Inside the workgroup the WAVEFRONTS SPLIT THE KEYS:
// wave w takes the 32-key blocks w, w+4, ... of the split and all query rows, so
// no K/V tile is shared between waves and nothing in the main loop goes through
// LDS.  The four partial (max, sum, O) states are merged through LDS at the end.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, wave64).  Scores are computed
// transposed, S^T = K Q^T (A = 16 keys x 32 features, B = 32 features x 16
// queries), so that a lane ends up holding 8 consecutive keys of one query
// column; those 8 probabilities are exactly the 8 k-slots that lane must supply
// as B operand of O^T += V^T P^T (A = 16 features x 32 keys).  For that to work
// the two 16-key score tiles of a 32-key block interleave the keys in groups of
// four (tile A: keys 0-3, 8-11, 16-19, 24-27; tile B: the others), which costs
// nothing because a K row is addressed per lane anyway.  V pages are stored
// feature-major, so the V^T operand is one 16-byte load per lane; K rows are
// token-major, one 16-byte load per lane and k-step.  The head features are
// consumed in the order (step, lane group) -> 8-feature chunk 4*step + group for
// both Q and K, so every K load instruction covers 64 contiguous bytes per key.
//
// Softmax runs in the log2 domain with the scale folded into the exponent's FMA.
// The running maximum is only moved (and O rescaled) when it would grow by more
// than 2^8; until then probabilities are at most 256, which fp32 accumulation
// and bf16's fp32-sized exponent hold without loss.
//
// Only blocks that need a mask go a slower way: the ragged last block of the
// cached prefix (scores masked, V operand zeroed past the end) and the step's
// own R new rows (mask generated in registers from ancestor bit sets and stream
// ranges; V rows, which are token-major there, transposed through a per-wave
// LDS tile).
#include "ss_msa.h"

namespace ss {

constexpr float kLazyLog2 = 8.0f;

// key (0..31) that row m of score tile X holds inside a 32-key block
SS_DEV int block_key(int m, int X) { return 8 * (m >> 2) + (m & 3) + 4 * X; }

SS_DEV bf16x8 as_bf16x8(uintx4 u) { return __builtin_bit_cast(bf16x8, u); }

SS_DEV uintx4 ld16(const uint16_t* p) { return *reinterpret_cast<const uintx4*>(p); }

struct NoMask {
  SS_DEV bool operator()(int, int, int) const { return true; }
  static constexpr bool kMasked = false;
};

// ragged last block of the cached prefix: key offset 8*lg + 4*X + i must lie before the end
struct TailMask {
  int tail, lg;
  static constexpr bool kMasked = true;
  SS_DEV bool operator()(int, int X, int i) const { return 8 * lg + 4 * X + i < tail; }
};

// the step's own rows: tree + stream visibility of query tile t's row against new key c0 + offset
template <int NQT>
struct NewMask {
  const RowVis (&vis)[NQT];
  int c0, lg, R, T;
  static constexpr bool kMasked = true;
  SS_DEV bool operator()(int t, int X, int i) const {
    const int col = c0 + 8 * lg + 4 * X + i;
    return (col < R) & row_sees(vis[t], col, T);
  }
};

// One 32-key block against all query tiles of the workgroup.
// Qs: the query operands in LDS, one 16-byte entry per (query tile, k-step, lane).
template <int D, int NQT, class Mask>
SS_DEV void attend_block(const bf16x8 (&Kr)[2][D / 32], const bf16x8 (&Vr)[D / 16], const uintx4* Qs, int lane,
                         floatx4 (&O)[D / 16][NQT], float (&m)[NQT], float (&l)[NQT], float c, Mask mask) {
  constexpr int KS = D / 32, DT = D / 16;
  // The query operands are re-read from LDS for every block.  Hiding the lane
  // offset from the optimiser keeps it from hoisting those reads out of the key
  // loop into 16*NQT long-lived registers.
  asm volatile("" : "+v"(lane));
  floatx4 S[2][NQT];
#pragma unroll
  for (int X = 0; X < 2; ++X)
#pragma unroll
    for (int t = 0; t < NQT; ++t) S[X][t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int t = 0; t < NQT; ++t) {
      const bf16x8 qop = as_bf16x8(Qs[(t * KS + ks) * 64 + lane]);
#pragma unroll
      for (int X = 0; X < 2; ++X) S[X][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Kr[X][ks], qop, S[X][t], 0, 0, 0);
    }

  bf16x8 P[NQT];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    if (Mask::kMasked) {
#pragma unroll
      for (int X = 0; X < 2; ++X)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float sv = S[X][t][i];
          S[X][t][i] = mask(t, X, i) ? sv : -INFINITY;
        }
    }
    float mx = fmaxf(fmaxf(fmaxf(S[0][t][0], S[0][t][1]), fmaxf(S[0][t][2], S[0][t][3])),
                     fmaxf(fmaxf(S[1][t][0], S[1][t][1]), fmaxf(S[1][t][2], S[1][t][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (__any((mx - m[t]) * c > kLazyLog2)) {
      const float m_new = fmaxf(m[t], mx);
      const float alpha = __builtin_amdgcn_exp2f((m[t] - m_new) * c);
      l[t] *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt][t] *= alpha;
      m[t] = m_new;
    }
    const float mc = m[t] * c;
    float ps = 0.f;
#pragma unroll
    for (int X = 0; X < 2; ++X)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(S[X][t][i], c, -mc));
        ps += p;
        P[t][4 * X + i] = (__bf16)p;
      }
    l[t] += ps;
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int t = 0; t < NQT; ++t) O[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Vr[dt], P[t], O[dt][t], 0, 0, 0);
}

template <int D, int NQT>
__global__ __launch_bounds__(256, 1) void msa_bf16_kernel(MsaArgs a) {
  constexpr int KS = D / 32, DT = D / 16, QROWS = 16 * NQT;
  constexpr int STAGE_BYTES = 4 * 32 * D * 2;            // per-wave V tiles of the new rows
  constexpr int MERGE_BYTES = 2 * DT * NQT * 64 * 16;    // two wave-sized O buffers
  constexpr int BUF_BYTES = STAGE_BYTES > MERGE_BYTES ? STAGE_BYTES : MERGE_BYTES;

  __shared__ int pt[4096];
  __shared__ int par[SS_MAX_T];
  __shared__ uint64_t anc[SS_MAX_T];
  __shared__ float m_sh[4][QROWS];
  __shared__ float l_sh[4][QROWS];
  __shared__ __attribute__((aligned(16))) unsigned char buf[BUF_BYTES];
  __shared__ uintx4 Qs[NQT * KS * 64];

  // ---- which piece of work: XCD-aware order.  Workgroup ids go round-robin over
  // the 8 XCDs, so ids that are equal mod 8 share an L2: the query chunks of one
  // (sequence, KV head, split) are given such ids and read K/V through one L2.
  const int G = a.B * a.Hkv * a.n_splits;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int qc = slot % a.n_qc;
  const int group = (slot / a.n_qc) * 8 + xcd;
  if (group >= G) return;
  const int s = group % a.n_splits;
  const int hk = (group / a.n_splits) % a.Hkv;
  const int b = group / (a.n_splits * a.Hkv);

  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lq = lane & 15, lg = lane >> 4;
  const int R = a.R, T = a.T, F = a.g * R;
  const int L = clamp_len(a.seq_lens[b], a);
  const int n_active = active_splits(L, a);
  if (s >= n_active) return;
  const bool is_last = (s == n_active - 1);
  const int k0 = s * a.split_keys;
  const int k1 = max(k0, min(L, k0 + a.split_keys));
  const float c = a.scale_log2;

  const uint16_t* q = (const uint16_t*)a.q;
  const uint16_t* k_new = (const uint16_t*)a.k_new;
  const uint16_t* v_new = (const uint16_t*)a.v_new;
  const uint16_t* k_cache = (const uint16_t*)a.k_cache;
  const uint16_t* v_cache = (const uint16_t*)a.v_cache;

  // ---- page ids of this split -> LDS (clamped), tree -> ancestor sets
  const int lp0 = k0 >> a.page_shift;
  const int npg = (k1 - k0 + a.page - 1) >> a.page_shift;
  for (int i = tid; i < npg; i += 256) {
    const int pg = a.block_table[(size_t)b * a.max_pages + lp0 + i];
    pt[i] = min(max(pg, 0), a.num_pages - 1);
  }
  if (tid < T) par[tid] = clamp_parent(a.parent[(size_t)b * T + tid], tid);
  __syncthreads();
  compute_anc(par, T, anc, tid);
  __syncthreads();

  // ---- query operands -> LDS in MFMA B-operand order (shared by the four waves: every
  // wave multiplies all query rows), and per-row visibility of the step's own keys
  for (int e = tid; e < NQT * KS * 64; e += 256) {
    const int t = e / (KS * 64), ks = (e >> 6) % KS, ln = e & 63;
    const int f = qc * QROWS + 16 * t + (ln & 15);
    uintx4 u = uintx4{0u, 0u, 0u, 0u};
    if (f < F) u = ld16(q + (((size_t)b * R + f % R) * a.H + hk * a.g + f / R) * D + (4 * ks + (ln >> 4)) * 8);
    Qs[e] = u;
  }
  RowVis vis[NQT];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int f = qc * QROWS + 16 * t + lq;
    vis[t] = make_row_vis(f < F ? f % R : 0, T, a.gamma, anc, (a.flags & SS_STREAM_EXCLUDE_SELF) != 0);
  }
  __syncthreads();

  floatx4 O[DT][NQT];
  float m[NQT], l[NQT];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    m[t] = -1e30f;
    l[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  bf16x8 Kr[2][KS], Vr[DT];
  const size_t k_page_stride = (size_t)a.Hkv * a.page * D;  // elements per physical page
  const int pmask = a.page - 1;

  auto load_k = [&](int kb) {
    const int key = kb + block_key(lq, 0);  // tile B's key is 4 further, on the same page
    const int pg = pt[(key >> a.page_shift) - lp0];
    const uint16_t* kp = k_cache + (size_t)pg * k_page_stride + ((size_t)hk * a.page + (key & pmask)) * D + lg * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Kr[0][ks] = as_bf16x8(ld16(kp + 32 * ks));
      Kr[1][ks] = as_bf16x8(ld16(kp + 4 * D + 32 * ks));
    }
  };
  auto load_v = [&](int kb) {
    const int key = kb + 8 * lg;
    const int pg = pt[(key >> a.page_shift) - lp0];
    const uint16_t* vp = v_cache + (size_t)pg * k_page_stride + ((size_t)hk * D + lq) * a.page + (key & pmask);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) Vr[dt] = as_bf16x8(ld16(vp + (size_t)16 * dt * a.page));
  };

  // ---- full 32-key blocks of the cached prefix: no mask, loads one block ahead,
  // K reloaded as soon as the scores are done, V as soon as P.V is done
  const int n_full = (k1 - k0) >> 5;
  if (w < n_full) {
    load_k(k0 + 32 * w);
    load_v(k0 + 32 * w);
  }
  for (int j = w; j < n_full; j += 4) {
    const bool more = (j + 4) < n_full;
    bf16x8 Kc[2][KS], Vc[DT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Kc[0][ks] = Kr[0][ks];
      Kc[1][ks] = Kr[1][ks];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) Vc[dt] = Vr[dt];
    if (more) {
      load_k(k0 + 32 * (j + 4));
      load_v(k0 + 32 * (j + 4));
    }
    attend_block<D, NQT>(Kc, Vc, Qs, lane, O, m, l, c, NoMask{});
  }

  // ---- blocks that need a mask, dealt round-robin to the waves after the full blocks
  const int tail = (k1 - k0) & 31;
  const int n_new_blocks = is_last ? (R + 31) >> 5 : 0;
  int unit = n_full;
  if (tail) {
    if ((unit & 3) == w) {
      const int kb = k0 + 32 * n_full;
#pragma unroll
      for (int X = 0; X < 2; ++X) {
        const int key = kb + min(block_key(lq, X), tail - 1);
        const int pg = pt[(key >> a.page_shift) - lp0];
        const uint16_t* kp = k_cache + (size_t)pg * k_page_stride + ((size_t)hk * a.page + (key & pmask)) * D + lg * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Kr[X][ks] = as_bf16x8(ld16(kp + 32 * ks));
      }
      {
        // the lane's 8 keys start at 8*lg; nv of them exist.  Address a chunk that
        // exists, then zero what lies past the end so that 0 * garbage cannot be NaN.
        const int nv = min(max(tail - 8 * lg, 0), 8);
        const int key = kb + (nv > 0 ? 8 * lg : ((tail - 1) & ~7));
        const int pg = pt[(key >> a.page_shift) - lp0];
        const uint16_t* vp = v_cache + (size_t)pg * k_page_stride + ((size_t)hk * D + lq) * a.page + (key & pmask);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uintx4 u = ld16(vp + (size_t)16 * dt * a.page);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t keep = nv >= 2 * e + 2 ? 0xffffffffu : (nv == 2 * e + 1 ? 0x0000ffffu : 0u);
            u[e] &= keep;
          }
          Vr[dt] = as_bf16x8(u);
        }
      }
      attend_block<D, NQT>(Kr, Vr, Qs, lane, O, m, l, c, TailMask{tail, lg});
    }
    ++unit;
  }
  for (int nb = 0; nb < n_new_blocks; ++nb, ++unit) {
    if ((unit & 3) != w) continue;
    const int c0 = 32 * nb;
#pragma unroll
    for (int X = 0; X < 2; ++X) {
      const int row = min(c0 + block_key(lq, X), R - 1);
      const uint16_t* kp = k_new + (((size_t)b * R + row) * a.Hkv + hk) * D + lg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) Kr[X][ks] = as_bf16x8(ld16(kp + 32 * ks));
    }
    // V rows are token-major here: stage the 32 rows in this wave's LDS tile, then gather columns
    uint16_t* vst = reinterpret_cast<uint16_t*>(buf) + w * 32 * D;
#pragma unroll
    for (int n = 0; n < DT; ++n) {
      const int id = lane + 64 * n;
      const int row = id / (D / 8), ch = id % (D / 8);
      const int src = min(c0 + row, R - 1);
      *reinterpret_cast<uintx4*>(vst + row * D + ch * 8) =
          ld16(v_new + (((size_t)b * R + src) * a.Hkv + hk) * D + ch * 8);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      uintx4 u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t lo = vst[(8 * lg + 2 * e) * D + 16 * dt + lq];
        const uint32_t hi = vst[(8 * lg + 2 * e + 1) * D + 16 * dt + lq];
        u[e] = lo | (hi << 16);
      }
      Vr[dt] = as_bf16x8(u);
    }
    __builtin_amdgcn_wave_barrier();
    attend_block<D, NQT>(Kr, Vr, Qs, lane, O, m, l, c, NewMask<NQT>{vis, c0, lg, R, T});
  }

  // ---- merge the four waves.  First agree on a common maximum per query and
  // bring every wave's sum and O to it, then add the O's pairwise through LDS.
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    l[t] += __shfl_xor(l[t], 16, 64);
    l[t] += __shfl_xor(l[t], 32, 64);
  }
  __syncthreads();  // all waves are done with the staging tiles in buf
  if (lg == 0) {
#pragma unroll
    for (int t = 0; t < NQT; ++t) {
      m_sh[w][16 * t + lq] = m[t];
      l_sh[w][16 * t + lq] = l[t];
    }
  }
  __syncthreads();
  float mw[NQT], lw[NQT];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int qi = 16 * t + lq;
    const float mm = fmaxf(fmaxf(m_sh[0][qi], m_sh[1][qi]), fmaxf(m_sh[2][qi], m_sh[3][qi]));
    float ll = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) ll += l_sh[ww][qi] * __builtin_amdgcn_exp2f((m_sh[ww][qi] - mm) * c);
    const float fac = __builtin_amdgcn_exp2f((m[t] - mm) * c);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt][t] *= fac;
    mw[t] = mm;
    lw[t] = ll;
  }
  floatx4* obuf = reinterpret_cast<floatx4*>(buf);
  constexpr int WAVE_TILES = DT * NQT * 64;
  if (w >= 2) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int t = 0; t < NQT; ++t) obuf[(w - 2) * WAVE_TILES + (dt * NQT + t) * 64 + lane] = O[dt][t];
  }
  __syncthreads();
  if (w < 2) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int t = 0; t < NQT; ++t) O[dt][t] += obuf[w * WAVE_TILES + (dt * NQT + t) * 64 + lane];
  }
  __syncthreads();
  if (w == 1) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int t = 0; t < NQT; ++t) obuf[(dt * NQT + t) * 64 + lane] = O[dt][t];
  }
  __syncthreads();
  if (w != 0) return;

  // ---- wave 0 finishes: normalise and store.  A lane holds features 16*dt+4*lg..+3 of query 16*t+lq.
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int f = qc * QROWS + 16 * t + lq;
    if (f >= F) continue;
    const int hg = f / R, r = f % R, h = hk * a.g + hg;
    const float inv = lw[t] > 0.f ? 1.f / lw[t] : 0.f;
    if (a.n_splits == 1) {
      uint16_t* op = (uint16_t*)a.out + (((size_t)b * R + r) * a.H + h) * D + 4 * lg;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const floatx4 v = (O[dt][t] + obuf[(dt * NQT + t) * 64 + lane]) * inv;
        *reinterpret_cast<uintx2*>(op + 16 * dt) = uintx2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
      }
    } else {
      const size_t pr = (((size_t)b * a.H + h) * a.n_splits + s) * R + r;
      float* op = a.part_o + pr * D + 4 * lg;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        *reinterpret_cast<floatx4*>(op + 16 * dt) = (O[dt][t] + obuf[(dt * NQT + t) * 64 + lane]) * inv;
      if (lg == 0) a.part_lse[pr] = mw[t] * c + __log2f(lw[t]);
    }
  }
}

int msa_bf16_rows_per_chunk(int F) {
  if (F <= 80) return 16 * ceil_div(F < 1 ? 1 : F, 16);
  int best = 80, best_pad = ceil_div(F, 80) * 80 - F;
  const int cands[2] = {64, 48};
  for (int cnd : cands) {
    const int pad = ceil_div(F, cnd) * cnd - F;
    if (pad < best_pad) {
      best = cnd;
      best_pad = pad;
    }
  }
  return best;
}

template <int D>
static int launch_d(const MsaArgs& a, hipStream_t stream) {
  const int rows = msa_bf16_rows_per_chunk(a.g * a.R);
  const int G = a.B * a.Hkv * a.n_splits;
  const long wgs = (long)ceil_div(G, 8) * 8 * a.n_qc;
  SS_REQUIRE(wgs <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "ss_msa_attention: grid too large");
  dim3 grid((unsigned)wgs), block(256);
  switch (rows / 16) {
    case 1: hipLaunchKernelGGL((msa_bf16_kernel<D, 1>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((msa_bf16_kernel<D, 2>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((msa_bf16_kernel<D, 3>), grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((msa_bf16_kernel<D, 4>), grid, block, 0, stream, a); break;
    case 5: hipLaunchKernelGGL((msa_bf16_kernel<D, 5>), grid, block, 0, stream, a); break;
    default: SS_FAIL(SS_ERR_UNSUPPORTED, "ss_msa_attention: bad row chunk %d", rows);
  }
  return check_launch("ss_msa_attention");
}

int launch_msa_bf16(const MsaArgs& a, hipStream_t stream) {
  if (a.D == 128) return launch_d<128>(a, stream);
  return launch_d<64>(a, stream);
}

}  // namespace ss
