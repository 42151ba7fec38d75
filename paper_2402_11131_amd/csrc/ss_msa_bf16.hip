// a2, bf16 path: multi-stream attention (Eq. 1 / Eq. 2) on the gfx950 matrix cores.
//
// Work split.  A workgroup owns one (sequence, KV head, split of the cached
// tokens, chunk of <= 80 folded query rows, or of 128 where a KV head has more
// than 80); the query heads of a GQA group are
// folded into the row dimension, so K and V are read once per KV head.  The
// workgroup consists of G groups of NW wavefronts.  Inside a group every wave
// owns ONE 16-row query tile (its Q operands, running max / sum and a 16 x D
// slice of O live in registers) and all NW waves walk the same sequence of
// 32-key units; the G groups take the units of the split round-robin and their
// partial (max, sum, O) states are merged through LDS at the end.  With 80 rows
// that is up to 3 groups x 5 waves = 15 waves per compute unit, with 128 rows 2 groups
// x 8 waves = 16, which is what hides the LDS, MFMA and exp latencies (no wave depends
// on long instruction-level overlap).
//
// Memory pipeline.  Every group has a ring of n_stages LDS stages (8 KB of K rows + 8 KB of V for D = 128).
// Blocks reach it by direct global -> LDS loads (16 bytes per lane, no staging register, counted in the issuing
// wave's vector-memory counter and completed in issue order); up to four waves of a group issue them, one 1 KB
// slot per instruction, n_stages - 1 blocks ahead.  An iteration waits (hand-written s_waitcnt) for its own
// block, one workgroup barrier publishes it and frees the stage consumed one iteration earlier, which the next
// block is then sent to.  Global addresses are chosen so that one K instruction covers whole 256-byte key rows
// (4 consecutive keys = 1 KB contiguous) and one V instruction one contiguous KB of a feature-major page; the
// XOR swizzles of the LDS tiles are applied on the source side, by the lane -> address mapping.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, wave64).  Scores are computed
// transposed, S^T = K Q^T (A = 16 keys x 32 features, B = 32 features x 16
// queries), so that a lane ends up holding 8 consecutive keys of one query
// column; those 8 probabilities are exactly the 8 k-slots that lane must supply
// as B operand of O^T += V^T P^T (A = 16 features x 32 keys).  For that to work
// the two 16-key score tiles of a unit interleave the keys in groups of four
// (tile 0: keys 0-3, 8-11, 16-19, 24-27; tile 1: the others).  V pages are stored
// feature-major, so a V^T operand is 16 contiguous bytes.  In LDS the K rows are
// row-major and the V tile is feature-major, both with their 16-byte chunks
// XOR-swizzled so that every operand read is bank-conflict free.  The head
// features are consumed in the order (step, lane group) -> chunk 4*step + group
// for both Q and K.
//
// Softmax runs in the log2 domain with the scale folded into the exponent's FMA.
// The running maximum is only moved (and O rescaled) when it would grow by more
// than 2^16; until then probabilities are at most 65536, which fp32 accumulation
// and bf16's fp32-sized exponent hold without loss.
//
// Three kinds of units: full blocks of the cached prefix (no mask), the ragged
// last block of the prefix (scores masked, V zeroed past the end so that
// 0 * garbage cannot produce NaN) and blocks of the step's own R new rows (mask
// generated in registers from ancestor bit sets and stream ranges; V rows are
// token-major there: they are staged row-major and read with the LDS transpose
// read ds_read_b64_tr_b16, which hands a lane 4 consecutive keys of one feature).
// The ragged block alone goes through registers (per-lane page lookups, clamped).
//
// Order of work.  The step's own rows belong to split 0, which every sequence has,
// and are scanned FIRST: their addresses do not depend on the page table, so they
// are loaded and computed while the table and then the first prefix block are on
// their way (two dependent memory round trips during which a workgroup has nothing
// else to do).  The full prefix blocks follow in the pipelined main loop, the
// ragged block (owned by whichever split holds the end of the sequence) comes last.
#include <stdlib.h>

#include <mutex>
#include <type_traits>

#include "ss_msa.h"

namespace ss {

// Stores and loads that are coherent at device scope by themselves (the sc1 bit: written through to, read from,
// the level all XCDs share), for the partial results the in-kernel split merge hands from one workgroup to
// another: no cache-wide write-back or invalidate is then needed around the arrival counter.
SS_DEV void st16_device(float* p, floatx4 v) { asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory"); }
SS_DEV void st4_device(float* p, float v) { asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory"); }
// lse and DT 16-byte pieces (64 bytes apart) of one partial row, as relaxed device-scope loads of 8 bytes each:
// the compiler knows them as loads, so they can be issued early and are waited for at their first use.
template <int DT>
SS_DEV void ld_row_device(const float* lse_p, const float* o_p, float& lse, floatx4 (&o)[DT]) {
  lse = __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned int*>(lse_p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const unsigned long long* p8 = reinterpret_cast<const unsigned long long*>(o_p + 16 * dt);
    const unsigned long long lo = __hip_atomic_load(p8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(p8 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    o[dt] = floatx4{__uint_as_float((unsigned int)lo), __uint_as_float((unsigned int)(lo >> 32)),
                    __uint_as_float((unsigned int)hi), __uint_as_float((unsigned int)(hi >> 32))};
  }
}
// Arrival counter of the in-kernel split merge, read and written at device scope.
SS_DEV unsigned int ld_counter_device(const unsigned int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
SS_DEV void st_counter_device(unsigned int* p, unsigned int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Maximum as one instruction: the median of (a, b, +inf).  fmaxf() on matrix-core results costs an extra
// instruction per operand (the compiler first quiets signalling NaNs), a fifth of all vector work in the softmax
// of a 32-key block.  `pinf` is +inf in a register the compiler cannot see through (it would turn the median back
// into that maximum).  A compiler builtin, not inline assembly: the wait states between a matrix instruction or a
// row swap and the first reader of its result are inserted by the compiler only for instructions it knows.
SS_DEV float vmax2(float a, float b, float pinf) { return __builtin_amdgcn_fmed3f(a, b, pinf); }
// Maximum over the four lanes l, l^16, l^32, l^48 (the lanes that share a query row), left in all four, by
// the row-swap instructions: rows of 16 lanes [r0 r1 r2 r3] and a copy become [r0 r0 r2 r2] and [r1 r1 r3 r3],
// then halves of 32 lanes likewise.  No trip through LDS, unlike a general lane shuffle.
SS_DEV float max_over_lane_groups(float x, float pinf) {
  const unsigned int u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned int v = __float_as_uint(vmax2(__uint_as_float(a[0]), __uint_as_float(a[1]), pinf));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return vmax2(__uint_as_float(b[0]), __uint_as_float(b[1]), pinf);
}

constexpr float kLazyLog2 = 16.0f;
constexpr int kMaxGroups = 4;  // wave groups per workgroup
constexpr int kMaxWaves = 16;  // waves per workgroup: 4 per SIMD leaves each wave 128 vector registers

// key (0..31) that row m of score tile X holds inside a 32-key unit
SS_DEV int block_key(int m, int X) { return 8 * (m >> 2) + (m & 3) + 4 * X; }
// XOR swizzle of a K row's 16-byte chunks inside an LDS stage.  An operand read takes one chunk of
// each of the 16 rows block_key(0..15, X) per LDS cycle (16 lanes, 64 banks of 4 bytes): the swizzle
// has to spread those 16 chunks over all 16 bank groups.  Rows of 256 bytes (D = 128) cover the banks
// once each, so the 16 rows need 16 different 4-bit values; rows of 128 bytes (D = 64) alternate
// between the two halves of the banks, so rows of equal parity need 8 different 3-bit values.
template <int D>
SS_DEV int k_swz(int row) {
  return D == 128 ? ((row & 3) | (((row >> 3) & 3) << 2)) : (((row >> 1) & 1) | (((row >> 3) & 3) << 1));
}

SS_DEV bf16x8 as_bf16x8(uintx4 u) { return __builtin_bit_cast(bf16x8, u); }
SS_DEV uintx4 ld16(const uint16_t* p) { return *reinterpret_cast<const uintx4*>(p); }
// The same with the streaming hint: the K/V cache is read once per call and should not displace anything in
// the L2 and the memory-side cache (measured: 9 % less kernel time on the 4096-token workloads).
template <bool STREAM>
SS_DEV uintx4 ld16_cache(const uint16_t* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(p));
  else return *reinterpret_cast<const uintx4*>(p);
}

// LDS transpose read.  Within each group of 16 lanes, lane j passes the address of 4 consecutive
// 16-bit elements In[j][0..3]; lane i receives Out[i][e] = In[4*e + (i >> 2)][i & 3].  With lane
// (i = feature, group) pointing at row (i >> 2) and columns 4*(i & 3).. of a row-major tile, it
// receives feature i of rows 0..3: four consecutive keys of one feature.
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;
SS_DEV uintx2 lds_read_tr16(const unsigned char* p) {
  const shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(uintx2, v);
}

// 16 bytes per lane from (sbase + voff) straight into LDS: lane l's piece lands at lds_addr + 16*l.  No
// staging register and no LDS store instruction; the load counts in the issuing wave's vector-memory
// counter and completes in issue order.  STREAM adds the streaming hint (data no other workgroup asks for).
template <bool STREAM>
SS_DEV void dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0 nt" ::"s"(sbase), "v"(voff), "s"(lds_addr) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(sbase), "v"(voff), "s"(lds_addr) : "memory", "m0");
}
// Waits until at most `units` blocks' worth of this wave's direct-to-LDS loads (LPB per block) are outstanding.
// The counter has 6 bits; a smaller number than asked for only waits longer.
template <int N>
SS_DEV void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N < 63 ? N : 63) : "memory");
}
template <int LPB>
SS_DEV void wait_vm_units(int units) {
  switch (units) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<LPB>(); break;
    case 2: wait_vmcnt<2 * LPB>(); break;
    case 3: wait_vmcnt<3 * LPB>(); break;
    case 4: wait_vmcnt<4 * LPB>(); break;
    case 5: wait_vmcnt<5 * LPB>(); break;
    case 6: wait_vmcnt<6 * LPB>(); break;
    case 7: wait_vmcnt<7 * LPB>(); break;
    case 8: wait_vmcnt<8 * LPB>(); break;
    case 9: wait_vmcnt<9 * LPB>(); break;
    case 10: wait_vmcnt<10 * LPB>(); break;
    case 11: wait_vmcnt<11 * LPB>(); break;
    case 12: wait_vmcnt<12 * LPB>(); break;
    case 13: wait_vmcnt<13 * LPB>(); break;
    case 14: wait_vmcnt<14 * LPB>(); break;
    default: wait_vmcnt<15 * LPB>(); break;
  }
}
constexpr int kMaxStages = 10;  // ring stages per wave group: at most kMaxStages - 1 blocks in flight per group

// NW = waves (query tiles) per group; it only fixes how the 1 KB load slots of a unit are dealt to
// the waves of a group.  The number of groups and the ring depth are launch parameters.
// STREAM: the cache is loaded with the streaming hint.  Right when a (sequence, KV head, split) has one row
// chunk, so that every byte of the cache is wanted by exactly one workgroup; with several row chunks (long GQA
// trees) the chunks share K/V through the L2 and the hint undoes that (measured: +25 % time).
template <int D, int NW, bool STREAM>
__global__ __launch_bounds__(64 * NW * (kMaxWaves / NW < kMaxGroups ? kMaxWaves / NW : kMaxGroups)) void msa_bf16_kernel(MsaArgs a, int n_groups, int n_stages) {
  constexpr int KS = D / 32, DT = D / 16;
  constexpr int K_BYTES = 32 * D * 2;          // K rows of a unit (V takes the same)
  constexpr int STAGE_BYTES = 2 * K_BYTES;
  constexpr int K_SLOTS = K_BYTES / 1024;      // 1 KB load slots of a unit's K rows (V: as many)
  constexpr int LW = NW >= 4 ? 4 : NW >= 2 ? 2 : 1;  // waves of a group that move data: divides K_SLOTS
  constexpr int KJ = K_SLOTS / LW;             // K slots per loading wave, and V slots per loading wave
  constexpr int LPB = 2 * KJ;                  // loads per block and loading wave
  constexpr int CPR = D / 8;                   // 16-byte chunks per K row
  constexpr int ROWS_PER_SLOT = 64 / CPR;
  constexpr int V_DBLK = K_SLOTS / 2;          // 32-feature blocks per 16-key half of the V tile
  constexpr int VHALF = D * 32;                // bytes of one 16-key half of the V tile: D feature rows of 32 bytes

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // smem: [n_groups][n_stages][STAGE_BYTES] ring stages, overlaid by the buffer of the final merge of the groups
  // ([n_groups - 1][NW][DT] KB); behind the larger of the two: par | anc | ml
  unsigned char* stages = smem;
  const int ring_bytes = n_groups * n_stages * STAGE_BYTES, merge_bytes = (n_groups - 1) * NW * DT * 1024;
  int* par = reinterpret_cast<int*>(smem + max(ring_bytes, merge_bytes));
  uint64_t* anc = reinterpret_cast<uint64_t*>(par + SS_MAX_T);
  float* ml = reinterpret_cast<float*>(anc + SS_MAX_T);  // [n_groups][NW][2][16]: max, sum per query

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

  // The wave index is made known to be wave-uniform, so that everything derived from it (unit, load
  // slots, base addresses) is computed on the scalar unit.
  const int tid = threadIdx.x, lane = tid & 63, lq = lane & 15, lg = lane >> 4;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = w / NW, wt = w % NW;  // wave group, query tile of this wave
  const int R = a.R, T = a.T, F = a.g * R;
  const int k0 = split_begin(s, a);     // this split's cached tokens are [k0, k1)
  const float c = a.scale_log2;

  const uint16_t* q = (const uint16_t*)a.q;
  const int32_t* my_table = a.block_table + (size_t)b * a.max_pages;
  const size_t page_stride = (size_t)a.Hkv * a.page * D;  // elements per physical page (K and V alike)
  const uint16_t* k_head = (const uint16_t*)a.k_cache + (size_t)hk * a.page * D;  // this head inside page 0
  const uint16_t* v_head = (const uint16_t*)a.v_cache + (size_t)hk * a.page * D;
  const int pmask = a.page - 1;

  unsigned char* my_stages = stages + (size_t)grp * n_stages * STAGE_BYTES;
  const uint32_t lds_stages = (uint32_t)(uintptr_t)my_stages;

  // ---- first round trip: page ids, sequence length, tree, queries.
  // Physical pages of the two 16-key halves of this group's main-loop units (equal for pages of 32
  // or 64 tokens; positions past the table are clamped, such units are never used).  Lane i of every
  // wave keeps the pair for loop iteration jbase + i; one gather serves 64 iterations and a page id
  // reaches the scalar unit through a lane read.
  // What is kept is the page's offset in the cache in units of 256 bytes (a page of one head is at least
  // 16 x 64 x 2 bytes, and 2^32 such units are 1 TB), so that the scalar unit needs a shift, not a 64-bit product.
  uint32_t tab_a = 0, tab_b = 0;
  const uint32_t page_units = (uint32_t)(page_stride / 128);
  const int key_cap = max(a.max_pages * a.page - 32, 0) & ~31;  // last 32-key block the table covers
  auto refill_pages = [&](int jbase) {
    const int kb = min(k0 + 32 * (grp + (jbase + lane) * n_groups), key_cap);
    tab_a = (uint32_t)min(max(my_table[kb >> a.page_shift], 0), a.num_pages - 1) * page_units;
    tab_b = (uint32_t)min(max(my_table[min((kb + 16) >> a.page_shift, a.max_pages - 1)], 0), a.num_pages - 1) * page_units;
  };
  refill_pages(0);
  const int L_raw = a.seq_lens[b];
  const int n_kept = kept_nodes(b, a);
  int par_v = tid < T ? clamp_parent(a.parent[(size_t)b * T + tid], tid) : 0;

  // this wave's query tile: MFMA B operands (lane (lq, lg) holds features 8*(4*ks+lg).. of folded query row f)
  // Rows of nodes that pruning removed are neither computed nor written: the folded row index runs over the
  // kept rows only (per query head the n_kept main rows, then the n_kept*gamma stream rows of those nodes), so
  // the kept rows fill the first row chunks and the workgroups of the others leave at once.
  const int R_kept = n_kept * (1 + a.gamma);
  if (qc * (16 * NW) >= a.g * R_kept) return;
  const int f = qc * (16 * NW) + 16 * wt + lq;
  const bool f_valid = f < a.g * R_kept;
  const int f_row = f_valid ? f % R_kept : 0;
  const int q_r = f_row < n_kept ? f_row : T + (f_row - n_kept), q_h = hk * a.g + (f_valid ? f / R_kept : 0);
  bf16x8 Qr[KS];
  {
    const uint16_t* qp = q + (((size_t)b * R + q_r) * a.H + q_h) * D + lg * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uintx4 u = uintx4{0u, 0u, 0u, 0u};
      if (f_valid) u = ld16(qp + 32 * ks);
      Qr[ks] = as_bf16x8(u);
    }
  }

  floatx4 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  // Running maximum, and the running sum of the probabilities as the matrix cores add it up: one more
  // instruction per block, a row of ones times P^T, instead of eight vector additions per lane; all four
  // entries of a lane hold the sum of its query row over all keys of the block (the bf16 probabilities that
  // also enter P V, so numerator and denominator round alike).
  float m_run = -1e30f;
  float nmc_run = 1e30f * c;             // -(m_run * c), kept beside m_run: one multiplication less per block
  const float lazy_thr = kLazyLog2 / c;  // the scale is positive: (mx - m_run) * c > 2^4 <=> mx - m_run > lazy_thr
  float m_lim = m_run + lazy_thr;        // scores above this move the maximum; kept beside it as well
  floatx4 Lacc = floatx4{0.f, 0.f, 0.f, 0.f};
  bf16x8 ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
  // Kept in four registers from here on: as a known constant the compiler would build it anew in every block.
  asm volatile("" : "+v"(ones));

  // ---- how a block reaches LDS.  A unit is moved in 1 KB slots, one direct-to-LDS load each: K slot sl
  // holds rows ROWS_PER_SLOT*sl + lane/CPR, the lane at chunk position p = lane%CPR fetching chunk
  // p ^ k_swz(row).  The V tile consists of two halves of 16 keys, each D feature rows of 32 bytes; V slot
  // s2 holds features dblk*32 + lane/2 of half s2 / V_DBLK (dblk = s2 % V_DBLK), the lane at position
  // lane&1 fetching the 8-key chunk (lane&1) ^ ((feature >> 3) & 1), which makes the 16-lane operand reads
  // (16 features x 16 bytes) hit 64 different banks.  In a feature-major page a slot is one contiguous KB.
  // The first LW waves of a group move the data: wave wt takes K slots and V slots wt + LW*j.
  const int ril = lane / CPR, pch = lane % CPR;
  const bool loader = wt < LW;
  const int wl = loader ? wt : 0;
  // Slot sl lies in the second 16-key half of the unit when sl >= K_SLOTS / 2 (K and V alike); its offset inside
  // the half is part of the lane's byte offset, so that a half has one scalar base.
  uint32_t k_voff[KJ], v_voff[KJ];  // per lane, bytes from the half's scalar base
  bool second[KJ];
#pragma unroll
  for (int j = 0; j < KJ; ++j) {
    const int sl = wl + LW * j, r0 = ROWS_PER_SLOT * sl;
    second[j] = sl >= K_SLOTS / 2;
    k_voff[j] = 2u * (uint32_t)((r0 & 15) * D + ril * D + ((pch ^ k_swz<D>(r0 + ril)) * 8));
    v_voff[j] = 2u * (uint32_t)((sl % V_DBLK) * 32 * a.page + (lane >> 1) * a.page + (((lane & 1) ^ ((lane >> 4) & 1)) * 8));
  }
  // operand reads: K row of score tile 0 (tile 1 is 4 rows further, same swizzle), chunk 4*ks + lg; V:
  // feature 16*dt + lq, keys 8*lg .. 8*lg+7
  const int rr0 = block_key(lq, 0);
  int k_rd[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_rd[ks] = rr0 * (2 * D) + (((4 * ks + lg) ^ k_swz<D>(rr0)) * 16);
  const int v_rd = K_BYTES + (lg >> 1) * VHALF + lq * 32 + (((lg & 1) ^ ((lq >> 3) & 1)) * 16);

  // Main-loop unit u (a full block of the prefix) -> LDS stage at st_addr: scalar base per half.
  auto dma_main = [&](int u, uint32_t pg_a, uint32_t pg_b, uint32_t st_addr) {
    const int kb = k0 + 32 * u;
    const uint32_t o_a = (uint32_t)(kb & pmask), o_b = (uint32_t)((kb + 16) & pmask);
    const size_t g_a = (size_t)pg_a << 8, g_b = (size_t)pg_b << 8;  // bytes
    const char* ka = (const char*)k_head + g_a + o_a * (2 * D);
    const char* kb2 = (const char*)k_head + g_b + o_b * (2 * D);
    const char* va = (const char*)v_head + g_a + 2 * o_a;
    const char* vb = (const char*)v_head + g_b + 2 * o_b;
    const uint32_t slot_addr = st_addr + (uint32_t)wl * 1024;
#pragma unroll
    for (int j = 0; j < KJ; ++j) dma16<STREAM>(second[j] ? kb2 : ka, k_voff[j], slot_addr + LW * j * 1024);
#pragma unroll
    for (int j = 0; j < KJ; ++j) dma16<STREAM>(second[j] ? vb : va, v_voff[j], slot_addr + K_BYTES + LW * j * 1024);
  };
  // Rows c0 .. c0+31 of the step's own block -> LDS stage at st_addr: K rows as above, V rows token-major
  // (row r at 2*D*r, chunk position p holding chunk p ^ 2*(r&3)) for the transposing operand read.  Rows past
  // R repeat the last one (they are masked).  The lane id is laundered so that none of this arithmetic is
  // kept in registers across the main loop.
  auto dma_new = [&](int c0, uint32_t st_addr) {
    int lane2 = lane;
    asm volatile("" : "+v"(lane2));
    const int ril2 = lane2 / CPR, pch2 = lane2 % CPR;
    const size_t head0 = ((size_t)b * R * a.Hkv + hk) * D;  // elements to row 0 of this sequence and head
    const uint16_t* kn = (const uint16_t*)a.k_new + head0;
    const uint16_t* vn = (const uint16_t*)a.v_new + head0;
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
      const int sl = wl + LW * j;
      const int rr = ROWS_PER_SLOT * sl + ril2;
      const uint32_t row_off = (uint32_t)min(c0 + rr, R - 1) * (uint32_t)(a.Hkv * D * 2);
      dma16<false>(kn, row_off + (uint32_t)((pch2 ^ k_swz<D>(rr)) * 16), st_addr + sl * 1024);
      dma16<false>(vn, row_off + (uint32_t)((pch2 ^ (2 * (rr & 3))) * 16), st_addr + K_BYTES + sl * 1024);
    }
  };

  // ---- the ragged last block of the prefix goes through registers (per-lane page lookups, clamped to
  // existing keys; what is read in excess is masked).  base = its first cached token, last = the last one.
  uintx4 stg[2 * KJ];
  auto load_ragged = [&](int base, int last) {
    int lane2 = lane;
    asm volatile("" : "+v"(lane2));
    const int ril2 = lane2 / CPR, pch2 = lane2 % CPR;
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
      const int sl = wl + LW * j;
      const int rr = ROWS_PER_SLOT * sl + ril2;
      const int key = min(base + rr, last);
      const int pg = min(max(my_table[key >> a.page_shift], 0), a.num_pages - 1);
      const uint16_t* ksrc = k_head + (size_t)pg * page_stride + (size_t)(key & pmask) * D;
      const int half = sl / V_DBLK, dblk = sl % V_DBLK;
      const int vkey = min(base + 16 * half + (lane2 & 1) * 8, last & ~7);
      const int vpg = min(max(my_table[vkey >> a.page_shift], 0), a.num_pages - 1);
      const uint16_t* vsrc = v_head + (size_t)vpg * page_stride + (size_t)(dblk * 32 + (lane2 >> 1)) * a.page + (vkey & pmask);
      stg[j] = ld16(ksrc + ((pch2 ^ k_swz<D>(rr)) * 8));
      stg[KJ + j] = ld16(vsrc);
    }
  };
  auto store_ragged = [&](unsigned char* st) {
    int lane2 = lane;
    asm volatile("" : "+v"(lane2));
#pragma unroll
    for (int j = 0; j < KJ; ++j) {
      const int sl = wl + LW * j;
      *reinterpret_cast<uintx4*>(st + sl * 1024 + lane2 * 16) = stg[j];
      const int half = sl / V_DBLK, fr = (sl % V_DBLK) * 32 + (lane2 >> 1);
      *reinterpret_cast<uintx4*>(st + K_BYTES + half * VHALF + fr * 32 + (((lane2 & 1) ^ ((fr >> 3) & 1)) * 16)) = stg[KJ + j];
    }
  };

  // Split 0's first block of the step's own rows travels with the first round trip (its addresses need
  // nothing from memory), into the last ring stage, which the main loop does not fill before its first barrier.
  const bool has_new = s == 0;  // every sequence has a split 0
  const int n_new_units = (R + 31) >> 5;
  const uint32_t new_stage = lds_stages + (uint32_t)(n_stages - 1) * STAGE_BYTES;
  if (has_new && loader && grp < n_new_units) dma_new(32 * grp, new_stage);

  // ---- what there is to do.  The sequence length arrives with the page ids.
  const int L = clamp_len(L_raw, a);
  const int n_active = active_splits(L, a);
  if (s >= n_active) return;
  const int k1 = max(k0, min(L, k0 + split_len(s, a)));
  // Units of this split: full 32-key blocks of the prefix (ring-buffered main loop of n_main iterations,
  // one block per group and iteration; group grp has n_mine of them) and its ragged last block.
  const int n_full = (k1 - k0) >> 5;
  const int tail = (k1 - k0) & 31;
  const int n_main = (n_full + n_groups - 1) / n_groups;
  const int n_mine = grp < n_full ? (n_full - grp + n_groups - 1) / n_groups : 0;

  // Everything loaded so far is waited for here, before the first direct-to-LDS load is issued: the
  // compiler knows nothing of those loads, and a wait it places later for one of its own would wait for
  // all of them too.
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(tab_a), "+v"(tab_b), "+v"(par_v)::"memory");
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(Qr[ks]));

  // ---- second round trip: the first blocks of the prefix.
  const int n_pre = min(n_mine, n_stages - 1);
  if (loader)
    for (int i = 0; i < n_pre; ++i)
      dma_main(grp + i * n_groups, __builtin_amdgcn_readlane(tab_a, i), __builtin_amdgcn_readlane(tab_b, i),
               lds_stages + (uint32_t)i * STAGE_BYTES);
  if (tid < T) par[tid] = par_v;
  __syncthreads();
  compute_anc(par, T, anc, tid);
  __syncthreads();

  float pinf = INFINITY;  // see vmax2
  asm volatile("" : "+s"(pinf));
  const RowVis no_vis = RowVis{0, 0, 0};
  // One unit out of an LDS stage: scores, softmax update, O += P V.  `full` (a compile-time flag) is
  // the unmasked main-loop flavour; otherwise the unit is the ragged block of the prefix, or (is_new)
  // rows c0.. of the step's own block and `vis` tells which of those this lane's query row may see.
  auto compute = [&](auto full, bool is_new, int c0, const unsigned char* st, const RowVis& vis) {
    constexpr bool FULL = decltype(full)::value;
    // The masked flavours recompute their lane-dependent offsets on every call (the lane id is
    // laundered) instead of keeping them in registers across the loops.
    int ln = lane;
    if (!FULL) asm volatile("" : "+v"(ln));
    const int mq = ln & 15, mg = ln >> 4;
    // ---- scores S^T = K Q^T
    floatx4 S[2];
#pragma unroll
    for (int X = 0; X < 2; ++X) {
      floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uintx4 kop = *reinterpret_cast<const uintx4*>(st + k_rd[ks] + X * (8 * D));
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kop), Qr[ks], acc, 0, 0, 0);
      }
      S[X] = acc;
    }
    // ---- mask (only the ragged prefix block and the new rows)
    if (!FULL) {
#pragma unroll
      for (int X = 0; X < 2; ++X)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int off = 8 * mg + 4 * X + i;
          const bool see_tail = off < tail;
          const bool see_new = (c0 + off < R) & row_sees(vis, c0 + off, T);
          const float sv = S[X][i];
          S[X][i] = (is_new ? see_new : see_tail) ? sv : -INFINITY;
        }
    }
    // ---- online softmax (log2 domain, lazy rescale), probabilities to bf16
    // The maximum of a query row lies in four lanes; whether any row of the wave has to move its running
    // maximum can be told from the lanes' own eight scores, so the exchange between the lanes happens only then.
    const float mx8 = vmax2(vmax2(vmax2(S[0][0], S[0][1], pinf), vmax2(S[0][2], S[0][3], pinf), pinf),
                            vmax2(vmax2(S[1][0], S[1][1], pinf), vmax2(S[1][2], S[1][3], pinf), pinf), pinf);
    if (__any(mx8 > m_lim)) {
      const float mx = max_over_lane_groups(mx8, pinf);
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      Lacc *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt] *= alpha;
      m_run = m_new;
      nmc_run = -(m_new * c);
      m_lim = m_new + lazy_thr;
    }
    bf16x8 P;
#pragma unroll
    for (int X = 0; X < 2; ++X)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        P[4 * X + i] = (__bf16)__builtin_amdgcn_exp2f(fmaf(S[X][i], c, nmc_run));
      }
    Lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, P, Lacc, 0, 0, 0);
    // ---- O^T += V^T P^T
    if (FULL) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const uintx4 vv = *reinterpret_cast<const uintx4*>(st + v_rd + dt * 512);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), P, O[dt], 0, 0, 0);
      }
    } else if (!is_new) {
      const int nv = min(max(tail - 8 * mg, 0), 8);  // how many of this lane's 8 tokens exist
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        uintx4 vv = *reinterpret_cast<const uintx4*>(st + v_rd + dt * 512);
#pragma unroll
        for (int e = 0; e < 4; ++e) vv[e] &= nv >= 2 * e + 2 ? 0xffffffffu : (nv == 2 * e + 1 ? 0x0000ffffu : 0u);
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), P, O[dt], 0, 0, 0);
      }
    } else {
      const unsigned char* vb = st + K_BYTES;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        uintx2 half[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int row = 8 * mg + 4 * hh + (mq >> 2);  // keys 8*lg + 4*hh .. +3 reach this lane
          const int ch = 2 * dt + ((mq & 3) >> 1);      // 16-byte chunk with features 16*dt + 4*(lq&3)..
          half[hh] = lds_read_tr16(vb + row * (2 * D) + ((ch ^ (2 * (row & 3))) * 16) + (mq & 1) * 8);
        }
        const uintx4 vv = uintx4{half[0][0], half[0][1], half[1][0], half[1][1]};
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), P, O[dt], 0, 0, 0);
      }
    }
  };

  // ---- the step's own rows (split 0), one block per group and round, while the first prefix blocks
  // are on their way.
  if (has_new) {
    const RowVis vis = make_row_vis(q_r, T, a.gamma, anc, (a.flags & SS_STREAM_EXCLUDE_SELF) != 0);
    for (int jn = 0; jn * n_groups < n_new_units; ++jn) {
      const int un = jn * n_groups + grp;
      const bool mine = un < n_new_units;
      if (jn > 0) {
        __syncthreads();  // the previous round's block has been consumed
        if (loader && mine) dma_new(32 * un, new_stage);
      }
      // round 0: only the prefix blocks issued after it may still be in flight; later rounds: nothing
      if (loader && mine) wait_vm_units<LPB>(jn == 0 ? n_pre : 0);
      __syncthreads();
      if (mine) compute(std::false_type{}, true, 32 * un, my_stages + (size_t)(n_stages - 1) * STAGE_BYTES, vis);
    }
  }

  // ---- main loop over full blocks of the prefix.  Ring of n_stages stages per group, n_stages - 1 blocks
  // in flight: iteration `it` waits for its own block (loads complete in order), one barrier publishes it
  // and tells that the stage of iteration it - 1 has been consumed, which the block of iteration
  // it + n_stages - 1 then goes to.
  const bool rag_mine = tail != 0 && grp == 0;  // group 0 has a block in every iteration
  const int rag_base = k0 + 32 * n_full;
  if (n_main == 0 && rag_mine && loader) load_ragged(rag_base, k1 - 1);
  {
    int st_comp = 0, st_fill = n_stages - 1;  // ring positions of iteration it and of iteration it + n_stages - 1
    for (int it = 0; it < n_main; ++it) {
      if (loader && it < n_mine) wait_vm_units<LPB>(min(n_mine - 1 - it, n_stages - 2));
      __syncthreads();
      const int jl = it + n_stages - 1;
      if (loader && jl < n_mine) {
        if ((jl & 63) == 0) refill_pages(jl);
        dma_main(grp + jl * n_groups, __builtin_amdgcn_readlane(tab_a, jl & 63), __builtin_amdgcn_readlane(tab_b, jl & 63),
                 lds_stages + (uint32_t)st_fill * STAGE_BYTES);
      }
      if (it == n_main - 1 && rag_mine && loader) load_ragged(rag_base, k1 - 1);  // nothing else is in flight now
      if (it < n_mine) compute(std::true_type{}, false, 0, my_stages + (size_t)st_comp * STAGE_BYTES, no_vis);
      st_comp = st_comp + 1 == n_stages ? 0 : st_comp + 1;
      st_fill = st_fill + 1 == n_stages ? 0 : st_fill + 1;
    }
  }
  // ---- the ragged last block of the prefix (group 0), loaded while the last main-loop unit was computed
  if (tail != 0) {
    __syncthreads();  // the stages are free
    if (rag_mine && loader) store_ragged(my_stages);
    __syncthreads();
    if (rag_mine) compute(std::false_type{}, false, 0, my_stages, no_vis);
  }

  // ---- merge the groups.  Every wave reduces its sum over the four lane groups; groups > 0 leave
  // (max, sum, O) in LDS; group 0 brings everything to a common maximum, adds and stores.
  const bool split_launch = a.n_splits > 1;
  const bool merge_here = split_launch && a.arrive != nullptr && !(a.flags & SS_MSA_PARTIALS_ONLY);
  // In-kernel merge of two splits.  Every query tile of a split has an arrival counter.  A tile that finds
  // the other split's tile already arrived (or the sequence too short to have another split) takes that
  // split's partial rows from memory, folds them with what it holds in registers and writes the final rows.
  // Otherwise it stores its own partial rows, announces itself, and does the same only if the other tile
  // arrived in between.  Nothing waits for anything.  The counter is read early, before the wave groups are
  // merged, so that the other split's rows travel while that happens.
  unsigned int* ctr = nullptr;
  unsigned int early = 0;
  if (merge_here && grp == 0) {
    ctr = a.arrive + (((size_t)b * a.Hkv + hk) * a.n_qc + qc) * kArriveTiles + wt;
    // The address is the same in all lanes, but the compiler must not know: it would move the value to the
    // scalar unit at once, i.e. wait for this round trip here, in front of the merge of the groups.
    int zero = 0;
    asm volatile("" : "+v"(zero));
    early = ld_counter_device(ctr + zero);
  }
  float l_run = Lacc[0];  // already summed over the four lane groups
  floatx4* obuf = reinterpret_cast<floatx4*>(stages);  // [(grp-1)*NW + wt][DT][64]
  float* my_ml = ml + (grp * NW + wt) * 32;
  __syncthreads();  // every group is done with its stages (the merge buffer overlays them)
  if (grp > 0) {
    if (lg == 0) {
      my_ml[lq] = m_run;
      my_ml[16 + lq] = l_run;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) obuf[(((grp - 1) * NW + wt) * DT + dt) * 64 + lane] = O[dt];
  }
  __syncthreads();
  if (grp > 0) return;

  // rows of the other split, on their way during the merge of the groups
  const int s_other = 1 - s;
  early = __builtin_amdgcn_readfirstlane(early);
  const bool others_ready = merge_here && early + 1 == (unsigned)n_active;  // n_active is 1 or 2 here
  const bool prefetched = others_ready && n_active == 2 && f_valid;
  float l_other = -INFINITY;
  floatx4 o_other[DT];
  const size_t pr_other = (((size_t)b * a.H + q_h) * a.n_splits + s_other) * R + q_r;
  if (prefetched) ld_row_device<DT>(a.part_lse + pr_other, a.part_o + pr_other * D + 4 * lg, l_other, o_other);

  float mm = m_run;
  for (int g2 = 1; g2 < n_groups; ++g2) mm = fmaxf(mm, ml[(g2 * NW + wt) * 32 + lq]);
  {
    const float fac = __builtin_amdgcn_exp2f((m_run - mm) * c);
    l_run *= fac;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] *= fac;
  }
  for (int g2 = 1; g2 < n_groups; ++g2) {
    const float* oml = ml + (g2 * NW + wt) * 32;
    const float fac = __builtin_amdgcn_exp2f((oml[lq] - mm) * c);
    l_run += oml[16 + lq] * fac;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] += obuf[(((g2 - 1) * NW + wt) * DT + dt) * 64 + lane] * fac;
  }

  // ---- normalise and store.  A lane holds features 16*dt + 4*lg .. +3 of its query row.
  if (!f_valid) return;
  const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
  uint16_t* outp = (uint16_t*)a.out + (((size_t)b * R + q_r) * a.H + q_h) * D + 4 * lg;
  if (!split_launch) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const floatx4 v = O[dt] * inv;
      *reinterpret_cast<uintx2*>(outp + 16 * dt) = uintx2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    }
    return;
  }
  const size_t pr = (((size_t)b * a.H + q_h) * a.n_splits + s) * R + q_r;
  float* op = a.part_o + pr * D + 4 * lg;
  const float my_lse = mm * c + __log2f(l_run);
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] *= inv;
  if (!merge_here) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<floatx4*>(op + 16 * dt) = O[dt];
    if (lg == 0) a.part_lse[pr] = my_lse;
    return;
  }
  bool fold_now = others_ready;
  if (!others_ready) {
    // The splits run on different XCDs: the partial rows are stored coherently at device scope, and a
    // wave announces itself only when its stores have completed.
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) st16_device(op + 16 * dt, O[dt]);
    if (lg == 0) st4_device(a.part_lse + pr, my_lse);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's partial rows are where every XCD reads them
    unsigned int seen = 0;
    if (lane == 0) seen = atomicAdd(ctr, 1u);  // lane 0 holds the tile's first row: valid whenever any is
    seen = __builtin_amdgcn_readfirstlane(seen);
    fold_now = seen + 1 == (unsigned)n_active;
    if (fold_now) ld_row_device<DT>(a.part_lse + pr_other, a.part_o + pr_other * D + 4 * lg, l_other, o_other);
  }
  if (!fold_now) return;
  // the splits in index order with the arithmetic of the merge kernel, so that the result does not depend
  // on which split came last (its own rows are taken from registers, the other's from memory)
  floatx4 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  float M = -INFINITY, wsum = 0.f;
  auto fold = [&](float l2, const floatx4 (&o2)[DT]) {
    if (l2 > -INFINITY) {
      const float m_new = fmaxf(M, l2);
      const float keep = exp2f(M - m_new), w2 = exp2f(l2 - m_new);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) acc[dt] = merge_step(acc[dt], keep, o2[dt], w2);
      wsum = __builtin_fmaf(wsum, keep, w2);
      M = m_new;
    }
  };
  if (n_active == 2 && s_other == 0) fold(l_other, o_other);
  fold(my_lse, O);
  if (n_active == 2 && s_other == 1) fold(l_other, o_other);
  const float inv2 = wsum > 0.f ? 1.f / wsum : 0.f;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const floatx4 v = acc[dt] * inv2;
    *reinterpret_cast<uintx2*>(outp + 16 * dt) = uintx2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
  }
  if (lane == 0) st_counter_device(ctr, 0u);  // the next call finds the counters zero again
}

// Folded query rows one workgroup takes: a multiple of 16, at most 80 (five waves per wave group) where one chunk
// holds all rows.  With more rows (long GQA trees: the shapes bound by arithmetic and by the traffic from the L2,
// since every row chunk of a KV head fetches all of its K/V) the chunk that pads the rows least wins among 128
// (eight waves per group, two groups), 80, 64 and 48, the larger one on a tie: 640 rows are 5 chunks of 128
// (5.4 GB through the compute units' L1s on c5) rather than 8 of 80 (8.7 GB).
int msa_bf16_rows_per_chunk(int F) {
  if (F <= 80) return 16 * ceil_div(F < 1 ? 1 : F, 16);
  int best = 128, best_pad = ceil_div(F, 128) * 128 - F;
  const int cands[3] = {80, 64, 48};
  for (int cnd : cands) {
    const int pad = ceil_div(F, cnd) * cnd - F;
    if (pad < best_pad) {
      best = cnd;
      best_pad = pad;
    }
  }
  return best;
}

// Wave groups per workgroup for NW query tiles and ring stages per group: what the plan asks for (or the
// SS_MSA_GROUPS / SS_MSA_STAGES tuning overrides, read once), as far as kMaxWaves waves, the LDS of a compute
// unit and the 6-bit load counter allow (lpb = loads per block of a loading wave).
static int env_int_once(const char* name, int lo, int hi) {
  const char* e = getenv(name);
  const int v = e ? atoi(e) : 0;
  return (v >= lo && v <= hi) ? v : 0;
}
static int groups_for(int nw, int wanted) {
  static const int forced = env_int_once("SS_MSA_GROUPS", 1, kMaxGroups);
  int cap = kMaxWaves / nw;
  if (cap > kMaxGroups) cap = kMaxGroups;
  int g = forced ? forced : wanted;
  if (g > cap) g = cap;
  return g < 1 ? 1 : g;
}
static int stages_for(int n_groups, int wanted, size_t stage_bytes, int lpb) {
  static const int forced = env_int_once("SS_MSA_STAGES", 2, kMaxStages);
  int n = forced ? forced : wanted;
  if (n > kMaxStages) n = kMaxStages;
  while (n > 2 && ((size_t)n_groups * n * stage_bytes > 144 * 1024 || (n - 1) * lpb > 60)) --n;
  return n < 2 ? 2 : n;
}

template <int D, int NW, bool STREAM>
static int launch_dns(const MsaArgs& a, hipStream_t stream) {
  const int n_groups = groups_for(NW, a.groups);
  const int G = a.B * a.Hkv * a.n_splits;
  const long wgs = (long)ceil_div(G, 8) * 8 * a.n_qc;
  SS_REQUIRE(wgs <= 0x7fffffffL, SS_ERR_UNSUPPORTED, "ss_msa_attention: grid too large");
  const size_t stage_bytes = 2 * 32 * D * 2;
  constexpr int lw = NW >= 4 ? 4 : NW >= 2 ? 2 : 1;
  const int n_stages = stages_for(n_groups, a.stages, stage_bytes, 2 * (32 * D * 2 / 1024) / lw);
  const size_t merge_bytes = (size_t)(n_groups - 1) * NW * (D / 16) * 64 * 16;
  size_t lds = (size_t)n_groups * n_stages * stage_bytes;
  if (merge_bytes > lds) lds = merge_bytes;
  lds += SS_MAX_T * 4 + SS_MAX_T * 8 + (size_t)n_groups * NW * 32 * 4;
  SS_REQUIRE(lds <= 160 * 1024, SS_ERR_UNSUPPORTED, "ss_msa_attention: %zu bytes of LDS needed", lds);
  auto kern = msa_bf16_kernel<D, NW, STREAM>;
  static std::once_flag attr_once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [&]() {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  });
  if (attr_err != hipSuccess)
    SS_FAIL(SS_ERR_HIP, "ss_msa_attention: hipFuncSetAttribute: %s", hipGetErrorString(attr_err));
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(64 * NW * n_groups), lds, stream, a, n_groups, n_stages);
  return check_launch("ss_msa_attention");
}

template <int D, int NW>
static int launch_dn(const MsaArgs& a, hipStream_t stream) {
  return a.n_qc == 1 ? launch_dns<D, NW, true>(a, stream) : launch_dns<D, NW, false>(a, stream);
}

template <int D>
static int launch_d(const MsaArgs& a, hipStream_t stream) {
  const int rows = msa_bf16_rows_per_chunk(a.g * a.R);
  switch (rows / 16) {
    case 1: return launch_dn<D, 1>(a, stream);
    case 2: return launch_dn<D, 2>(a, stream);
    case 3: return launch_dn<D, 3>(a, stream);
    case 4: return launch_dn<D, 4>(a, stream);
    case 5: return launch_dn<D, 5>(a, stream);
    case 8: return launch_dn<D, 8>(a, stream);
    default: SS_FAIL(SS_ERR_UNSUPPORTED, "ss_msa_attention: bad row chunk %d", rows);
  }
}

int launch_msa_bf16(const MsaArgs& a, hipStream_t stream) {
  if (a.D == 128) return launch_d<128>(a, stream);
  return launch_d<64>(a, stream);
}

}  // namespace ss
