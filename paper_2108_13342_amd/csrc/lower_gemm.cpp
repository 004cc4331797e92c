// Contraction kernels: a block anchored on MatMul, with index-only prologues folded into the
// operand address functions and the block's One-to-One / Reorganize / Shuffle successors run as
// an epilogue on the accumulator tile (paper Sec. 4.4.1: fusing GEMM with a Shuffle-typed
// operator maps each GEMM output element to the destination that operator decides).
//
// Kernel shape (gfx950): 256 threads = 4 wavefronts in a 2x2 grid over a BM x BN output tile, each
// wavefront accumulating (BM/2)x(BN/2) with 32x32 MFMA tiles (v_mfma_f32_32x32x16 f16/bf16,
// v_mfma_f32_32x32x2 f32), fp32 accumulators.  Operand tiles go global -> registers -> LDS with
// the next tile's global loads in flight during the current tile's MFMAs.  LDS holds both
// operands K-contiguous so every fragment is one 16-byte read; an operand that is contiguous
// along M or N instead is transposed 8x8 in registers on its way into LDS.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>

#include "lower_ctx.hpp"

namespace dnnf {

int64_t stride_of(const Affine& a, int atom) {
  auto it = a.stride.find(atom);
  return it == a.stride.end() ? 0 : it->second;
}

std::string gemm_offset_fn(const LowerCtx& c, const std::string& name, const std::vector<int>& atoms, const Affine& a) {
  std::vector<std::pair<int64_t, int64_t>> es;   // (extent, stride), adjacent compatible atoms merged
  for (int at : atoms) {
    int64_t e = c.atom_extent[at], s = stride_of(a, at);
    if (!es.empty() && es.back().second == s * e) { es.back().first *= e; es.back().second = s; }
    else es.push_back({e, s});
  }
  std::ostringstream o;
  // the operand's constant offset (a Slice or Split in front of it) rides on the batch term, which every tile adds once
  const bool is_batch = name.size() > 6 && name.compare(name.size() - 6, 6, "_batch") == 0;
  o << "DEV idx_t " << name << "(idx_t x) {\n  idx_t off = " << (is_batch ? a.offset : 0) << ";\n";
  for (int k = (int)es.size() - 1; k >= 0; k--) {
    if (k == 0) o << "  off += x * (idx_t)" << es[k].second << ";\n";
    else {
      o << "  off += (x % " << es[k].first << ") * (idx_t)" << es[k].second << ";\n";
      o << "  x /= " << es[k].first << ";\n";
    }
  }
  o << "  return off;\n}\n";
  return o.str();
}

void decl_digits(std::ostringstream& os, const LowerCtx& c, const std::vector<int>& atoms_major_minor,
                 const std::string& counter, const std::string& ind, const std::string& tag) {
  std::string rem = counter;
  for (int k = (int)atoms_major_minor.size() - 1; k >= 0; k--) {
    int a = atoms_major_minor[k];
    int64_t e = c.atom_extent[a];
    if (k == 0) os << ind << "const idx_t a" << a << " = " << rem << ";\n";
    else {
      os << ind << "const idx_t a" << a << " = " << rem << " % " << e << ";\n";
      os << ind << "const idx_t " << tag << a << " = " << rem << " / " << e << ";\n";
      rem = tag + std::to_string(a);
    }
  }
}

namespace {
#define offset_fn gemm_offset_fn
// The fixed, hand-written part of the kernel.  Everything block-specific enters through macros
// and the generated functions offA_*/offB_*/epilogue().
const char* kGemmBody = R"KRN(
#define NT (64 * WAVES_M * WAVES_N * WAVES_K)                // threads per workgroup
#if ELEM_BYTES == 2
#define VEC 8
typedef u16x8 vec_t;
#else
#define VEC 4
typedef f32x4 vec_t;
#endif
#ifdef DMA
#define LDK BK                                              // tiles filled straight from global memory are not padded
#else
#define LDK (BK + VEC)
#endif
#define WTM (BM / WAVES_M)
#define WTN (BN / WAVES_N)
#define TM (WTM / 32)
#define TN (WTN / 32)
// Row-aligned stores (EPI_RA = elements per 16-byte vector): the destination rows are contiguous along the columns but
// their starts are not 16-byte aligned (an odd row length).  Every row of the accumulator slab is then shifted by the
// distance of its first column from a 16-byte boundary of the destination, so that whole groups of the slab are whole
// aligned vectors of the destination; only the row's first and last group (8 or 4 elements together) are stored
// element by element, in a short pass of their own.
#if defined(EPI_RA) && WAVES_K == 1 && !defined(EPI_T)
#define RA 1
#else
#define RA 0
#endif
#ifdef EPI_T
#define CLD (BN + 1)                                        // slab read down its columns: an odd pitch spreads the banks
#elif RA
#define CLD (BN + EPI_RA + 4)                               // room for the shift
#else
#define CLD (BN + 4)                                        // row pitch of the fp32 accumulator slab (16-byte aligned rows)
#endif
#ifdef CONV_DIRECT
#define CD_NK (2 * CD_J * CD_TAPS)                          // K values of one wavefront's share: CD_J channel pairs x taps
#define CD_SEG ((CD_NK + 63) / 64)                          // 64-lane segments of a row of the slice
#define CD_S (CD_SEG * 64 + 1)                              // row pitch of its filter slice in LDS
#define AB_BYTES (4 * WAVES_K * 32 * CD_S)
#else
#define AB_BYTES ((int)sizeof(elem_t) * NBUF * (BM + BN) * LDK)
#endif
// The epilogue parks the accumulators in an fp32 slab, one group of accumulator-tile rows per pass: pass p takes the
// tiles i in [p * EPI_IR, (p + 1) * EPI_IR) of every wavefront, so all wavefronts store at once and the slab holds
// SR = WAVES_M * EPI_IR * 32 rows of the output tile.  EPI_IR is the largest divisor of TM whose slab fits the LDS
// share the operand tiles leave this workgroup anyway (the share of as many workgroups as the operand tiles allow per
// compute unit), so fewer, larger passes are taken where they cost no occupancy.
#define CS1_BYTES (4 * WAVES_K * WAVES_M * 32 * CLD)
#define LDS_SHARE (AB_BYTES >= 81920 ? 155648 : AB_BYTES >= 53248 ? 79872 : AB_BYTES >= 40960 ? 53248 : AB_BYTES >= 32768 ? 40960 : AB_BYTES)
#define EPI_IR ((TM % 8 == 0 && 8 * CS1_BYTES <= LDS_SHARE) ? 8 : (TM % 4 == 0 && 4 * CS1_BYTES <= LDS_SHARE) ? 4 : (TM % 2 == 0 && 2 * CS1_BYTES <= LDS_SHARE) ? 2 : 1)
#define SR (WAVES_M * EPI_IR * 32)
#define CS_BYTES (EPI_IR * CS1_BYTES)
#define SMEM_MAIN (((AB_BYTES > CS_BYTES ? AB_BYTES : CS_BYTES) + 15) / 16 * 16)
// row of the output tile that slab row sl of pass p holds
#define SLAB_ROW(p, sl) (((sl) / (EPI_IR * 32)) * WTM + ((p) * EPI_IR + ((sl) / 32) % EPI_IR) * 32 + (sl) % 32)

DEV vec_t vzero() { vec_t v; for (int i = 0; i < VEC; ++i) v[i] = 0; return v; }
// the transposing B loader may use narrower column vectors (B_CVEC elements) when the columns are only
// contiguous or aligned in shorter runs
#ifndef B_CVEC
#define B_CVEC VEC
#endif
#if ELEM_BYTES == 2
typedef unsigned short cvec_t __attribute__((ext_vector_type(B_CVEC)));      // bit containers, like vec_t
#else
typedef float cvec_t __attribute__((ext_vector_type(B_CVEC)));
#endif
DEV cvec_t cvzero() { cvec_t v; for (int i = 0; i < B_CVEC; ++i) v[i] = 0; return v; }

// ---- operand tile loaders: global -> registers
// DIRECT: the operand is contiguous along K; one 16-byte vector per (row, k-octet).
#define A_DIRECT_N ((BM * BK / VEC + NT - 1) / NT)
#define B_DIRECT_N ((BN * BK / VEC + NT - 1) / NT)
// TRANSPOSE: contiguous along the row/col axis; one thread owns a VEC x VEC sub-block.
#define A_TR_N ((BM * BK / (VEC * VEC) + NT - 1) / NT)
#define B_TR_N ((BN * BK / (B_CVEC * VEC) + NT - 1) / NT)       // B_CVEC columns x VEC k per thread
// SCALAR: anything else, element by element.
#define A_SC_N ((BM * BK + NT - 1) / NT)
#define B_SC_N ((BN * BK + NT - 1) / NT)

#if B_MODE == 3 && NT % BN != 0
#error "gathering loader: the tile width must divide the workgroup size"
#endif
#if defined(EPI_ROWNORM) && (BN < GN || WAVES_K != 1)
#error "row normalisation in the epilogue: one column tile must hold the whole row"
#endif
#if defined(CONV_DIRECT) && (BM != 32 || BN != 32 || WAVES_M != 1 || WAVES_N != 1 || ELEM_BYTES != 4)
#error "direct convolution loop: one 32 x 32 fp32 tile per workgroup"
#endif
extern "C" __global__ __launch_bounds__(NT) void KNAME(KPARAMS) {
  // one LDS allocation: the operand tiles during the main loop, an fp32 accumulator slab afterwards
#ifdef W_PREFETCH_LINES
#define W_PF_BYTES 256
#else
#define W_PF_BYTES 0
#endif
  __shared__ __attribute__((aligned(16))) char smem[SMEM_MAIN + (RA ? 4 * BM : 0) + W_PF_BYTES];
  typedef elem_t (*tile_a_t)[BM][LDK];
  typedef elem_t (*tile_b_t)[BN][LDK];
  const tile_a_t As = (tile_a_t)smem;
  const tile_b_t Bs = (tile_b_t)(smem + sizeof(elem_t) * NBUF * BM * LDK);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // WAVES_M x WAVES_N wavefronts tile the block's output; WAVES_K > 1 splits each K tile between
  // wavefronts that share an output tile (small problems: more workgroups, shorter MFMA chains)
  const int wk = wave / (WAVES_M * WAVES_N), wmn = wave % (WAVES_M * WAVES_N);
  const int wm = wmn / WAVES_N, wn = wmn % WAVES_N;
  // Workgroups are dealt round-robin to the 8 XCDs; renumber so that neighbouring tiles (which
  // share operand rows/columns) run on the same XCD and hit in its L2.
  idx_t bid = blockIdx.x;
  {
    const idx_t nb = gridDim.x, per = nb / 8, rem = nb % 8;
    const idx_t x = bid % 8, q = bid / 8;
    bid = x * per + (x < rem ? x : rem) + q;
  }
  const idx_t tiles_n = (GN + BN - 1) / BN, tiles_m = (GM + BM - 1) / BM;
  const idx_t z = bid / (tiles_m * tiles_n);
  idx_t t = bid % (tiles_m * tiles_n);
  // groups of 8 tile-rows walk the N direction together
  const idx_t grp = 8 * tiles_n, g0 = (t / grp) * 8;
  const idx_t gsz = (tiles_m - g0) < 8 ? (tiles_m - g0) : 8;
  const idx_t tile_m = g0 + (t % grp) % gsz, tile_n = (t % grp) / gsz;
  const idx_t row0 = tile_m * BM, col0 = tile_n * BN;
  const elem_t* __restrict__ Ab = PA + offA_batch(z);
  const elem_t* __restrict__ Bb = PB + offB_batch(z);
#ifdef W_PREFETCH_LINES
  // The weight operand was last read an inference ago and comes from memory; fetched K tile by K tile, every step of
  // every workgroup's loop would wait for a memory round trip of its own.  Instead the workgroups of each XCD touch
  // the whole matrix between them before anything else (one 4-byte load per 128-byte line, landing in a spare piece of
  // LDS that nobody reads), so all of it is on its way into that XCD's L2 while the first tiles are being loaded.
  {
    typedef __attribute__((address_space(1))) const void* wpf_gptr_t;
    typedef __attribute__((address_space(3))) void* wpf_lptr_t;
    const idx_t nx = (gridDim.x + 7) / 8, j = blockIdx.x / 8;
    const idx_t per = (W_PREFETCH_LINES + nx - 1) / nx;
    for (idx_t i = tid; i < per; i += NT) {
      const idx_t line = j * per + i;
      if (line < W_PREFETCH_LINES)
        __builtin_amdgcn_global_load_lds((wpf_gptr_t)((const char*)W_PREFETCH_PTR + line * 128),
                                         (wpf_lptr_t)(smem + SMEM_MAIN + (RA ? 4 * BM : 0)), 4, 0, 0);
    }
  }
#endif

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

  // Edge handling: rows and columns beyond the problem are clamped to the last valid one (their
  // products land in accumulator elements the epilogue never stores), so only a ragged K needs
  // zero fill.  Every test below folds to a constant when the tile sizes divide the problem, which
  // leaves the main loop free of branches and lets loads of later tiles stay in flight.
#define FULL_K (GK % BK == 0)
#define ROW_A(r) ((GM % BM == 0) ? (idx_t)(row0 + (r)) : ((row0 + (r)) < GM ? (idx_t)(row0 + (r)) : (idx_t)(GM - 1)))
#define COL_B(r) ((GN % BN == 0) ? (idx_t)(col0 + (r)) : ((col0 + (r)) < GN ? (idx_t)(col0 + (r)) : (idx_t)(GN - 1)))
#define WHOLE(n) ((n) % NT == 0)                         // every thread has work in each pass over n items
  const int nk = (GK + BK - 1) / BK;
#ifdef DMA
  // Both operands contiguous along K, 16-bit, K a multiple of BK: the tiles go from global memory straight
  // into LDS (global_load_lds, 16 bytes per lane), past the registers and without LDS store instructions.
  // One such instruction of a wavefront fills 1 KB of consecutive LDS: 64 / (BK / 8) rows of BK elements,
  // unpadded.  Fragment reads stay conflict-free because the 16-byte chunks of a row are stored permuted:
  // chunk c of row r sits in slot c ^ f(r), f(r) = (r ^ (r >> 3)) & (BK / 8 - 1) -- any 8 or 16
  // consecutive rows then meet different banks at the same c.  The permutation costs nothing: each lane
  // simply fetches the global chunk that belongs in its slot.
#define CPR (BK / VEC)                                   // 16-byte chunks per tile row
#define SWZ(r) ((((r) ^ ((r) >> 3))) & (CPR - 1))
  idx_t ra_off[A_DIRECT_N], rb_off[B_DIRECT_N];
  int ra_k[A_DIRECT_N], rb_k[B_DIRECT_N];
#pragma unroll
  for (int i = 0; i < A_DIRECT_N; ++i) {
    const int v = tid + i * NT, r = v / CPR;
    ra_off[i] = offA_row(ROW_A(r));
    ra_k[i] = ((v % CPR) ^ SWZ(r)) * VEC;
  }
#pragma unroll
  for (int i = 0; i < B_DIRECT_N; ++i) {
    const int v = tid + i * NT, r = v / CPR;
    rb_off[i] = offB_col(COL_B(r));
    rb_k[i] = ((v % CPR) ^ SWZ(r)) * VEC;
  }
  typedef __attribute__((address_space(1))) const void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto dma_load = [&](const int buf, const idx_t k0) {
#pragma unroll
    for (int i = 0; i < A_DIRECT_N; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(Ab + ra_off[i] + offA_k(k0 + ra_k[i])),
                                       (lptr_t)((char*)&As[buf][0][0] + (i * NT + wave * 64) * 16), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < B_DIRECT_N; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(Bb + rb_off[i] + offB_k(k0 + rb_k[i])),
                                       (lptr_t)((char*)&Bs[buf][0][0] + (i * NT + wave * 64) * 16), 16, 0, 0);
  };
  // Tile kt is multiplied from buffer kt & 1, one 16-deep K step at a time, with two sets of fragment registers:
  // while the MFMAs of step s run, the fragment reads of step s + 1 are already in flight (one wait per step,
  // after the MFMAs have been issued).  The reads that follow a tile's last step belong to the next tile: before
  // them the wavefront waits for its share of that tile's loads and meets the others (one barrier per tile), and
  // since every wavefront has then finished reading the current buffer, the loads of the tile after next start
  // into it right away - a whole tile of MFMA work ahead of their use.
#define KSTEPS (BK / 16)
  frag_t fa[2][TM], fb[2][TN];
  int fra[TM], frb[TN];                                    // row offsets of this lane's fragments, and the rows' swizzles
  int fsa[TM], fsb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) { const int r = wm * WTM + i * 32 + (lane & 31); fra[i] = r * LDK; fsa[i] = SWZ(r); }
#pragma unroll
  for (int j = 0; j < TN; ++j) { const int r = wn * WTN + j * 32 + (lane & 31); frb[j] = r * LDK; fsb[j] = SWZ(r); }
  auto frag_load = [&](const int buf, const int kk, const int set) {
    const int kc = kk * 2 + (lane >> 5);
    const elem_t* ab = &As[buf][0][0];
    const elem_t* bb = &Bs[buf][0][0];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[set][i] = __builtin_bit_cast(frag_t, *(const u16x8*)(ab + fra[i] + (kc ^ fsa[i]) * VEC));
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[set][j] = __builtin_bit_cast(frag_t, *(const u16x8*)(bb + frb[j] + (kc ^ fsb[j]) * VEC));
  };
#define LDS_WAIT() { __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_waitcnt(0xC07F); __builtin_amdgcn_sched_barrier(0); }   /* lgkmcnt(0) */
  // NBUF buffers: tile kt lives in buffer kt % NBUF and the loads run NBUF - 1 tiles ahead of the multiplications (two
  // buffers: one tile ahead - enough for operands that sit in the caches; three or four: for operands that another
  // kernel has just written, whose loads take several tile times to arrive).  A wavefront's loads complete in order, so
  // "tile kt + 1 has landed" is a wait until at most the loads of the tiles behind it are outstanding.
#define DMA_LPT (A_DIRECT_N + B_DIRECT_N)                 // load instructions per wavefront and tile
#define DMA_D (NBUF - 1)
#define VM_WAIT(n) { __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14)); __builtin_amdgcn_sched_barrier(0); }
  auto wait_tiles = [&](const int behind) {               // at most `behind` later tiles may still be in flight
    if (DMA_D >= 3 && behind >= 2) VM_WAIT(2 * DMA_LPT)
    else if (DMA_D >= 2 && behind == 1) VM_WAIT(DMA_LPT)
    else VM_WAIT(0)
  };
#pragma unroll
  for (int d = 0; d < DMA_D; ++d) if (d < nk) dma_load(d, (idx_t)d * BK);
  wait_tiles((nk < DMA_D ? nk : DMA_D) - 1);
  __syncthreads();
  frag_load(0, 0, 0);
  LDS_WAIT();
  // Wavefronts with at least as many matrix instructions as fragment reads per step (64x64 results and more): inside a
  // tile the reads of the next step are issued between the matrix instructions of the current one (one read after each
  // matrix instruction, in program order), and the K loop stays rolled - unrolled over a short constant K the address
  // arithmetic of every tile is hoisted and the registers spill.  Smaller wavefront tiles keep the block order (reads,
  // then matrix instructions), which measured faster for them.
#define N_MF (TM * TN)
#define N_RD (TM + TN)
#if N_MF >= N_RD || NBUF > 2
#define DMA_ROLLED 1
#endif
#if N_MF >= N_RD
#define DMA_INTERLEAVE 1
#endif
  int buf = 0;
#ifdef DMA_ROLLED
#pragma unroll 1
#endif
  for (int kt = 0; kt < nk; ++kt) {
    // everybody has left tile kt - 1 (the barrier that opened this tile): its buffer takes tile kt + NBUF - 1
    if (kt + DMA_D < nk) { int nb = buf + DMA_D; if (nb >= NBUF) nb -= NBUF; dma_load(nb, (idx_t)(kt + DMA_D) * BK); }
    int nxt = buf + 1; if (nxt >= NBUF) nxt = 0;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      if (kk + 1 < KSTEPS) frag_load(buf, kk + 1, (kk + 1) & 1);
      else if (kt + 1 < nk) {
        // this wavefront's share of tile kt + 1 is in LDS (the tiles up to min(kt + NBUF - 1, nk - 1) may stay in flight),
        const int last = kt + DMA_D < nk ? kt + DMA_D : nk - 1;
        wait_tiles(last - (kt + 1));
        __syncthreads();                                 // so is everybody's, and nobody reads `buf` any more
        __builtin_amdgcn_sched_barrier(0);
        frag_load(nxt, 0, 0);                            // KSTEPS is even: step 0 of the next tile uses set 0
      }
#ifndef DMA_INTERLEAVE
      __builtin_amdgcn_sched_barrier(0);
#else
      if (kk + 1 >= KSTEPS) __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = MFMA(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
#ifdef DMA_INTERLEAVE
      if (kk + 1 < KSTEPS) {
#pragma unroll
        for (int q = 0; q < N_RD; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one matrix instruction,
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // one LDS read
        }
        if (N_MF > N_RD) __builtin_amdgcn_sched_group_barrier(0x008, N_MF - N_RD, 0);
      }
#endif
      LDS_WAIT();
    }
    buf = nxt;
  }
#elif defined(CONV_DIRECT)
  // A convolution with too few 32 x 32 tiles to fill the chip is one memory round trip plus a chain of matrix
  // instructions, and staging K tile by K tile through LDS turns that into a chain of round trips.  Here K
  // (channel-major: k = channel * taps + tap) is split between the WAVES_K wavefronts of a tile by channels, and a
  // wavefront needs nobody else: every load of its share is in flight before its first multiply, and it meets the
  // others only to add the partial tiles up.
  //   pixels:  a lane fetches the values the matrix instructions take from it (lane & 31: column, lane >> 5: which
  //            of a step's two channels) straight into registers - neighbouring lanes are neighbouring pixels, and
  //            within a tap the window offset and the padding test are the same for every channel;
  //   filters: rows are contiguous along K, so lanes run along K for the loads (whole lines, row offsets in scalar
  //            registers) and the slice is turned through a private piece of LDS with an odd row pitch: the 32 rows
  //            of a fragment read then sit in 32 different banks.
  {
    const int cl = lane & 31, kh2 = lane >> 5;
    const gcol_t gcol = gather_col(COL_B(cl));
    const int wku = __builtin_amdgcn_readfirstlane(wk);     // the wavefront's index, in a scalar register
    float* Aw = (float*)smem + wku * 32 * CD_S;
    const idx_t kbase = (idx_t)wku * CD_NK;
    // (the pitch covers whole 64-lane segments, so loads and stores need no lane masks: lanes past the slice fetch its
    // first element again and park it in the padding)
    // The loads are issued segment by segment - a 64-wide piece of every filter row, then the pixels of the channel
    // pairs whose K values that piece completes - and the multiplications follow in the same order, so the matrix
    // instructions of the first channels run while the loads of the later ones are still in flight.
#define CD_JEND(sg) ((sg) + 1 >= CD_SEG ? CD_J : ((sg) + 1) * 64 / (2 * CD_TAPS))     /* channel pairs complete after segment sg */
    float av[CD_SEG][32];
    float fb[CD_TAPS][CD_J];
#pragma unroll
    for (int sg = 0; sg < CD_SEG; ++sg) {
      const unsigned kl = (unsigned)(sg * 64 + lane);
      const bool in_k = kl < CD_NK && ((WAVES_K * CD_NK == GK) || kbase + kl < GK);       // channels beyond the last: zero rows of K
#pragma unroll
      for (int r = 0; r < 32; ++r) {
        const float* __restrict__ rp = Ab + (offA_row(ROW_A(r)) + kbase);         // (the filter matrix is contiguous along K)
        const float a = rp[in_k ? kl : 0u];
        av[sg][r] = in_k ? a : 0.0f;
      }
#pragma unroll
      for (int j = (sg ? CD_JEND(sg - 1) : 0); j < CD_JEND(sg); ++j)
#pragma unroll
        for (int t = 0; t < CD_TAPS; ++t) {
          const int ch = (wku * CD_J + j) * 2 + kh2;
          const bool in_c = (WAVES_K * CD_NK == GK) || ch < CD_C;
          const float b = conv_direct_b(in_c ? ch : 0, t, gcol, KARGS);
          fb[t][j] = in_c ? b : 0.0f;
        }
    }
    const float* ar = Aw + cl * CD_S + kh2 * CD_TAPS;
#pragma unroll
    for (int sg = 0; sg < CD_SEG; ++sg) {
#pragma unroll
      for (int r = 0; r < 32; ++r) Aw[r * CD_S + sg * 64 + lane] = av[sg][r];
      // the slice is written and read by this wavefront alone, whose LDS operations complete in order
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = (sg ? CD_JEND(sg - 1) : 0); j < CD_JEND(sg); ++j)
#pragma unroll
        for (int t = 0; t < CD_TAPS; ++t)
          acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ar[2 * j * CD_TAPS + t], fb[t][j], acc[0][0], 0, 0, 0);
    }
  }
#else
#if A_MODE == 0
  vec_t ra[PF][A_DIRECT_N]; idx_t ra_off[A_DIRECT_N];
#pragma unroll
  for (int i = 0; i < A_DIRECT_N; ++i) {
    const int v = tid + i * NT, r = (WHOLE(BM * BK / VEC) || v < BM * BK / VEC) ? v / (BK / VEC) : 0;
    ra_off[i] = offA_row(ROW_A(r));
  }
#elif A_MODE == 1
  vec_t ra[PF][A_TR_N][VEC];
#else
  elem_t ra[PF][A_SC_N];
#endif
#if B_MODE == 0
  vec_t rb[PF][B_DIRECT_N]; idx_t rb_off[B_DIRECT_N];
#ifdef B_PROLOGUE
  idx_t rb_col[B_DIRECT_N];           // the generated operand prologue needs the column itself, not only its offset
#endif
#pragma unroll
  for (int i = 0; i < B_DIRECT_N; ++i) {
    const int v = tid + i * NT, r = (WHOLE(BN * BK / VEC) || v < BN * BK / VEC) ? v / (BK / VEC) : 0;
    rb_off[i] = offB_col(COL_B(r));
#ifdef B_PROLOGUE
    rb_col[i] = COL_B(r);
#endif
  }
#elif B_MODE == 4
  // channels-last convolution operand: K runs tap by tap, a 16-byte vector is VEC channels of one tap of one
  // column's pixel; the column is decoded once per thread, the tap once per vector
  vec_t rb[PF][B_DIRECT_N]; gcol_t rb_g[B_DIRECT_N];
#pragma unroll
  for (int i = 0; i < B_DIRECT_N; ++i) {
    const int v = tid + i * NT, r = (WHOLE(BN * BK / VEC) || v < BN * BK / VEC) ? v / (BK / VEC) : 0;
    rb_g[i] = gather_col(COL_B(r));
  }
#elif B_MODE == 1
  cvec_t rb[PF][B_TR_N][VEC];
#elif B_MODE == 3
  // BN divides the workgroup size: a thread gathers for one column throughout, decoded once
  elem_t rb[PF][B_SC_N];
  const gcol_t gcol = gather_col(COL_B(tid % BN));
#else
  elem_t rb[PF][B_SC_N];
#endif

  auto gload = [&](const int s_, idx_t k0) {
    if (k0 > (idx_t)(nk - 1) * BK) k0 = (idx_t)(nk - 1) * BK;      // past the end: re-read the last tile (never stored)
#if A_MODE == 0
#pragma unroll
    for (int i = 0; i < A_DIRECT_N; ++i) {
      const int v = tid + i * NT, kv = (v % (BK / VEC)) * VEC;
      ra[s_][i] = (FULL_K || k0 + kv < GK) ? *(const vec_t*)(Ab + ra_off[i] + offA_k(k0 + kv)) : vzero();
    }
#elif A_MODE == 1
#pragma unroll
    for (int i = 0; i < A_TR_N; ++i) {
      const int s = (WHOLE(BM * BK / (VEC * VEC)) || tid + i * NT < BM * BK / (VEC * VEC)) ? tid + i * NT : 0;
      const int kb8 = (s % (BK / VEC)) * VEC, rb8 = (s / (BK / VEC)) * VEC;      // see the store side for the lane order
      // a vector covers VEC consecutive rows: GM is a multiple of VEC in this mode, so it is inside or outside as a whole
      const idx_t ro = offA_row(ROW_A(rb8) / VEC * VEC);
#pragma unroll
      for (int j = 0; j < VEC; ++j)
        ra[s_][i][j] = (FULL_K || k0 + kb8 + j < GK) ? *(const vec_t*)(Ab + ro + offA_k(k0 + kb8 + j)) : vzero();
    }
#else
#pragma unroll
    for (int i = 0; i < A_SC_N; ++i) {
      const int e = (WHOLE(BM * BK) || tid + i * NT < BM * BK) ? tid + i * NT : 0, r = e / BK, k = e % BK;
      ra[s_][i] = (FULL_K || k0 + k < GK) ? Ab[offA_row(ROW_A(r)) + offA_k(k0 + k)] : (elem_t)0;
    }
#endif
#if B_MODE == 0
#pragma unroll
    for (int i = 0; i < B_DIRECT_N; ++i) {
      const int v = tid + i * NT, kv = (v % (BK / VEC)) * VEC;
      rb[s_][i] = (FULL_K || k0 + kv < GK) ? *(const vec_t*)(Bb + rb_off[i] + offB_k(k0 + kv)) : vzero();
    }
#elif B_MODE == 4
#pragma unroll
    for (int i = 0; i < B_DIRECT_N; ++i) {
      const int v = tid + i * NT, kv = (v % (BK / VEC)) * VEC;
      rb[s_][i] = (FULL_K || k0 + kv < GK) ? loadB_tap(k0 + kv, rb_g[i]) : vzero();
    }
#elif B_MODE == 1
#pragma unroll
    for (int i = 0; i < B_TR_N; ++i) {
      const int s = (WHOLE(BN * BK / (B_CVEC * VEC)) || tid + i * NT < BN * BK / (B_CVEC * VEC)) ? tid + i * NT : 0;
      const int kb8 = (s % (BK / VEC)) * VEC, cb8 = (s / (BK / VEC)) * B_CVEC;
      const idx_t co = offB_col(COL_B(cb8) / B_CVEC * B_CVEC);
#pragma unroll
      for (int j = 0; j < VEC; ++j)
        rb[s_][i][j] = (FULL_K || k0 + kb8 + j < GK) ? *(const cvec_t*)(Bb + co + offB_k(k0 + kb8 + j)) : cvzero();
    }
#elif B_MODE == 3
    // gathered operand (implicit im2col): lanes run along the columns so neighbouring pixels coalesce
#pragma unroll
    for (int i = 0; i < B_SC_N; ++i) {
      const int e = (WHOLE(BN * BK) || tid + i * NT < BN * BK) ? tid + i * NT : 0, r = e % BN, k = e / BN;
      rb[s_][i] = (FULL_K || k0 + k < GK) ? loadB_gather(Bb, k0 + k, gcol) : (elem_t)0;
    }
#else
#pragma unroll
    for (int i = 0; i < B_SC_N; ++i) {
      const int e = (WHOLE(BN * BK) || tid + i * NT < BN * BK) ? tid + i * NT : 0, r = e / BK, k = e % BK;
      rb[s_][i] = (FULL_K || k0 + k < GK) ? Bb[offB_col(COL_B(r)) + offB_k(k0 + k)] : (elem_t)0;
    }
#endif
  };

  // k0s: first K index of the tile being stored (used by an operand prologue only)
  auto lstore = [&](const int s_, const int buf, const idx_t k0s) {
#if A_MODE == 0
#pragma unroll
    for (int i = 0; i < A_DIRECT_N; ++i) {
      const int v = tid + i * NT, r = v / (BK / VEC), kv = (v % (BK / VEC)) * VEC;
      if (WHOLE(BM * BK / VEC) || v < BM * BK / VEC) *(vec_t*)&As[buf][r][kv] = ra[s_][i];
    }
#elif A_MODE == 1
#pragma unroll
    for (int i = 0; i < A_TR_N; ++i) {
      // neighbouring lanes own neighbouring K octets of the same rows: the BK / VEC lanes of a group write one whole
      // LDS row per store (every bank once), where lanes striding over rows would all start in the same banks
      const int s = tid + i * NT, kb8 = (s % (BK / VEC)) * VEC, rb8 = (s / (BK / VEC)) * VEC;
      if (WHOLE(BM * BK / (VEC * VEC)) || s < BM * BK / (VEC * VEC)) {
#pragma unroll
        for (int r = 0; r < VEC; ++r) {
          vec_t o;
#pragma unroll
          for (int j = 0; j < VEC; ++j) o[j] = ra[s_][i][j][r];
          *(vec_t*)&As[buf][rb8 + r][kb8] = o;
        }
      }
    }
#else
#pragma unroll
    for (int i = 0; i < A_SC_N; ++i) {
      const int e = tid + i * NT;
      if (WHOLE(BM * BK) || e < BM * BK) As[buf][e / BK][e % BK] = ra[s_][i];
    }
#endif
#if B_MODE == 0 || B_MODE == 4
#pragma unroll
    for (int i = 0; i < B_DIRECT_N; ++i) {
      const int v = tid + i * NT, r = v / (BK / VEC), kv = (v % (BK / VEC)) * VEC;
#ifdef B_PROLOGUE
      // One-to-One operators in front of the operand run here, on the way from registers to LDS, when the
      // vector's load has long landed; zero fill past the end of K stays zero
      if (WHOLE(BN * BK / VEC) || v < BN * BK / VEC)
        *(vec_t*)&Bs[buf][r][kv] = (FULL_K || k0s + kv < GK) ? b_prologue(rb[s_][i], rb_col[i], k0s + kv, KARGS) : rb[s_][i];
#else
      if (WHOLE(BN * BK / VEC) || v < BN * BK / VEC) *(vec_t*)&Bs[buf][r][kv] = rb[s_][i];
#endif
    }
#elif B_MODE == 1
#pragma unroll
    for (int i = 0; i < B_TR_N; ++i) {
      const int s = tid + i * NT, kb8 = (s % (BK / VEC)) * VEC, cb8 = (s / (BK / VEC)) * B_CVEC;
      if (WHOLE(BN * BK / (B_CVEC * VEC)) || s < BN * BK / (B_CVEC * VEC)) {
#pragma unroll
        for (int r = 0; r < B_CVEC; ++r) {
          vec_t o;
#pragma unroll
          for (int j = 0; j < VEC; ++j) o[j] = rb[s_][i][j][r];
          *(vec_t*)&Bs[buf][cb8 + r][kb8] = o;
        }
      }
    }
#elif B_MODE == 3
#pragma unroll
    for (int i = 0; i < B_SC_N; ++i) {
      const int e = tid + i * NT;
      if (WHOLE(BN * BK) || e < BN * BK) Bs[buf][e % BN][e / BN] = rb[s_][i];
    }
#else
#pragma unroll
    for (int i = 0; i < B_SC_N; ++i) {
      const int e = tid + i * NT;
      if (WHOLE(BN * BK) || e < BN * BK) Bs[buf][e / BK][e % BK] = rb[s_][i];
    }
#endif
  };

  auto compute_tile = [&](const int buf) {
#if ELEM_BYTES == 2
#pragma unroll
    for (int kq = 0; kq < BK / 16 / WAVES_K; ++kq) {
      const int kk = kq * WAVES_K + wk;
      frag_t fa[TM], fb[TN];
      const int kcol = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = __builtin_bit_cast(frag_t, *(const u16x8*)&As[buf][wm * WTM + i * 32 + (lane & 31)][kcol]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = __builtin_bit_cast(frag_t, *(const u16x8*)&Bs[buf][wn * WTN + j * 32 + (lane & 31)][kcol]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = MFMA(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
#else
#pragma unroll
    for (int kq = 0; kq < BK / 2 / WAVES_K; ++kq) {
      const int kk = kq * WAVES_K + wk;
      float fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = As[buf][wm * WTM + i * 32 + (lane & 31)][kk * 2 + (lane >> 5)];
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = Bs[buf][wn * WTN + j * 32 + (lane & 31)][kk * 2 + (lane >> 5)];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
#endif
  };

  // Software pipeline.  K tile t travels global -> register set t % PF -> LDS buffer t % NBUF.  PF
  // tiles are loaded ahead, so the latency of a tile's global loads overlaps PF - 1 tiles of MFMA work.
#pragma unroll
  for (int s = 0; s < PF; ++s) gload(s, (idx_t)s * BK);
  lstore(0, 0, 0);
  __syncthreads();
  for (int kt0 = 0; kt0 < nk; kt0 += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int kt = kt0 + u;
      if (kt < nk) {
        const int buf = NBUF == 2 ? (kt & 1) : 0;
        // a single register set is refilled while its tile (already in LDS) is multiplied
        if (PF == 1) gload(0, (idx_t)(kt + 1) * BK);
        compute_tile(buf);
#if NBUF == 2
        // the other buffer was last read one iteration ago and every wave has passed a barrier since
        if (kt + 1 < nk) lstore((u + 1) % PF, buf ^ 1, (idx_t)(kt + 1) * BK);
        if (PF > 1) gload(u, (idx_t)(kt + PF) * BK);
        __syncthreads();
#else
        __syncthreads();
        if (kt + 1 < nk) lstore((u + 1) % PF, 0, (idx_t)(kt + 1) * BK);
        if (PF > 1) gload(u, (idx_t)(kt + PF) * BK);
        __syncthreads();
#endif
      }
    }
  }
#endif   // DMA

  // Epilogue through LDS.  A lane of a 32x32 accumulator tile holds one column and 16 scattered
  // rows (element e: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32), which would store 2- or
  // 4-byte pieces of many rows.  Instead a slab of SR rows per pass is parked in LDS as fp32 and read back
  // with lanes running along the columns, so the generated epilogue sees consecutive columns in
  // consecutive lanes: its loads and stores coalesce into full lines, whatever index map the
  // block's Reorganize/Shuffle operators imposed on the destination.
  float* Cs = (float*)smem;
#if RA
  // per row of the tile: position of its first column inside a 16-byte group of the destination.  The table lies behind
  // the operand tiles, so it can be filled while other wavefronts still multiply; the slab loop's first barrier publishes it.
  int* rsh = (int*)(smem + SMEM_MAIN);
  for (int i = tid; i < BM; i += NT) rsh[i] = (row0 + i < GM) ? epi_row_pad(z, row0 + i, col0, KARGS) : 0;
#endif
#define COL_FIXED (NT % BN == 0)           // a thread then meets the same column in every pass
  const int cl = tid % BN;
  float colv[!COL_FIXED ? 1 : (NCOLV > 0 ? NCOLV : 1)];
  if (COL_FIXED && EPI_VEC == 1 && col0 + cl < GN) col_loads(col0 + cl, colv, KARGS);
#pragma unroll 1
  for (int h = 0; h < TM / EPI_IR; ++h) {
    __syncthreads();                        // operand tiles (or the previous slab) are no longer read
#pragma unroll
    for (int i = 0; i < TM; ++i)
      if (i / EPI_IR == h) {                // (a branch every wavefront takes the same way; the tile index stays static)
#if RA
        int sh[16];                         // shifts of the 16 rows this lane holds of the tile row: four runs of four rows
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const i32x4 s4 = *(const i32x4*)&rsh[wm * WTM + i * 32 + 8 * q + 4 * (lane >> 5)];
          sh[4 * q] = s4[0]; sh[4 * q + 1] = s4[1]; sh[4 * q + 2] = s4[2]; sh[4 * q + 3] = s4[3];
        }
#endif
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r32 = 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            const int sl = (wm * EPI_IR + i % EPI_IR) * 32 + r32;
#if RA
            Cs[sl * CLD + sh[e] + wn * WTN + j * 32 + (lane & 31)] = acc[i][j][e];
#else
            Cs[(wk * SR + sl) * CLD + wn * WTN + j * 32 + (lane & 31)] = acc[i][j][e];
#endif
          }
      }
    __syncthreads();
#ifdef EPI_ROWNORM
    // The tile holds whole rows of the product (one column tile).  Pass A runs the block's operators between the
    // product and the normalisation on every element (stores of their own included) and parks the value the
    // normalisation reads back in the slab; pass B gives every row to one wavefront: mean, centred second moment,
    // then the normalised value of each column goes through the operators behind the normalisation and is stored.
    for (int idx = tid; idx < SR * BN; idx += NT) {
      const int rl = idx / BN, c_l = idx % BN;
      const idx_t r = row0 + SLAB_ROW(h, rl);
      if (r < GM && c_l < GN) Cs[rl * CLD + c_l] = gn_value(z, r, c_l, Cs[rl * CLD + c_l], KARGS);
    }
    __syncthreads();
    for (int rl = wave; rl < SR; rl += NT / 64) {
      const idx_t r = row0 + SLAB_ROW(h, rl);
      if (r >= GM) continue;
      float s1 = 0.0f;
      for (int c_l = lane; c_l < GN; c_l += 64) s1 += Cs[rl * CLD + c_l];
      const float mean = dn_wave_sum(s1) * (1.0f / GN);
      float s2 = 0.0f;
      for (int c_l = lane; c_l < GN; c_l += 64) { const float dl = Cs[rl * CLD + c_l] - mean; s2 += dl * dl; }
      const float rstd = dn_div(1.0f, sqrtf(dn_wave_sum(s2) * (1.0f / GN) + NORM_EPS));
      for (int c_l = lane; c_l < GN; c_l += 64) gn_store((idx_t)z * GM + r, c_l, (Cs[rl * CLD + c_l] - mean) * rstd, KARGS);
    }
#elif RA
    // pass 1: the groups that are whole vectors of the destination (slab column q0 = tile column q0 - shift)
    // (a row that starts on a boundary has BN / EPI_RA whole groups from slab column 0 on, any other row one fewer from the
    // second group on: BN / EPI_RA slots per row either way)
#define RA_G (BN / EPI_RA)
#pragma unroll 2
    for (int idx = tid; idx < SR * RA_G; idx += NT) {
      const int rl = idx / RA_G;
      const int tr = SLAB_ROW(h, rl), pad = rsh[tr];
      const int q0 = (idx % RA_G + (pad ? 1 : 0)) * EPI_RA;
      const idx_t r = row0 + tr;
      const int c_l = q0 - pad;
      const idx_t c = col0 + c_l;
      if (r < GM && c_l + EPI_RA <= BN && c + EPI_RA <= GN) {
        float v[EPI_RA];
#pragma unroll
        for (int u = 0; u < EPI_RA; u += 4) {
          const f32x4 t4 = *(const f32x4*)&Cs[rl * CLD + q0 + u];
          v[u] = t4[0]; v[u + 1] = t4[1]; v[u + 2] = t4[2]; v[u + 3] = t4[3];
        }
        epilogue_ra(z, r, c, v, KARGS);
      }
    }
    // pass 2: what pass 1 left of every row - the columns in front of the first whole group and behind the last one
    // (at most 2 * EPI_RA - 2 of them), one element per thread
#pragma unroll 1
    for (int idx = tid; idx < SR * 2 * EPI_RA; idx += NT) {
      const int rl = idx / (2 * EPI_RA), u = idx % (2 * EPI_RA);
      const int tr = SLAB_ROW(h, rl);
      const idx_t r = row0 + tr;
      if (r >= GM) continue;
      const int pad = rsh[tr];
      // head: tile columns [0, first): first = (EPI_RA - pad) % EPI_RA.  tail: from the start of the last group that is not
      // whole (it runs past the tile or past the row's end) up to that end.
      const int first = (EPI_RA - pad) % EPI_RA;
      const int width = (GN - col0) < BN ? (int)(GN - col0) : BN;                    // valid columns of this tile
      const int last = first + (width - first) / EPI_RA * EPI_RA;                     // end of the whole groups
      const int cl = u < EPI_RA ? u : last + (u - EPI_RA);
      if (u < EPI_RA ? (cl < first && cl < width) : (cl >= first && cl < width)) {
        float cv[NCOLV > 0 ? NCOLV : 1];
        col_loads(col0 + cl, cv, KARGS);
        epilogue(z, r, col0 + cl, Cs[rl * CLD + pad + cl], cv, KARGS);
      }
    }
#elif EPI_VEC > 1 && defined(EPI_T)
    // the destinations are contiguous along the rows (a channels-last convolution result, a transposed
    // product): a thread takes EPI_VEC consecutive rows of one column, neighbouring lanes the next row
    // groups of the same column, so a wavefront's vector stores still cover whole lines
#pragma unroll 2
    for (int idx = tid; idx < (SR / EPI_VEC) * BN; idx += NT) {
      const int c_l = idx / (SR / EPI_VEC), rl = (idx % (SR / EPI_VEC)) * EPI_VEC;       // (EPI_VEC divides 32: the rows of a vector are consecutive rows of the output)
      float v[EPI_VEC];
#pragma unroll
      for (int u = 0; u < EPI_VEC; ++u) v[u] = Cs[(rl + u) * CLD + c_l];
#pragma unroll
      for (int q = 1; q < WAVES_K; ++q)
#pragma unroll
        for (int u = 0; u < EPI_VEC; ++u) v[u] += Cs[(q * SR + rl + u) * CLD + c_l];
      const idx_t r = row0 + SLAB_ROW(h, rl), c = col0 + c_l;
      if (r < GM && c < GN) epilogue_vec(z, c, r, v, KARGS);
    }
#elif EPI_VEC > 1
#pragma unroll 2
    for (int idx = tid; idx < SR * (BN / EPI_VEC); idx += NT) {
      const int rl = idx / (BN / EPI_VEC), c_l = (idx % (BN / EPI_VEC)) * EPI_VEC;
      float v[EPI_VEC];
#pragma unroll
      for (int u = 0; u < EPI_VEC; u += 4) {
        const f32x4 t4 = *(const f32x4*)&Cs[rl * CLD + c_l + u];
        v[u] = t4[0]; v[u + 1] = t4[1]; v[u + 2] = t4[2]; v[u + 3] = t4[3];
      }
#pragma unroll
      for (int q = 1; q < WAVES_K; ++q)
#pragma unroll
        for (int u = 0; u < EPI_VEC; ++u) v[u] += Cs[(q * SR + rl) * CLD + c_l + u];
      const idx_t r = row0 + SLAB_ROW(h, rl), c = col0 + c_l;
      if (r < GM && c < GN) epilogue_vec(z, r, c, v, KARGS);
    }
#else
#pragma unroll 8
    for (int idx = tid; idx < SR * BN; idx += NT) {
      const int rl = idx / BN, c_l = idx % BN;
      float v = Cs[rl * CLD + c_l];
#pragma unroll
      for (int q = 1; q < WAVES_K; ++q) v += Cs[(q * SR + rl) * CLD + c_l];
      const idx_t r = row0 + SLAB_ROW(h, rl), c = col0 + c_l;
      if (r < GM && c < GN) {
        if (!COL_FIXED) {
          float cv[NCOLV > 0 ? NCOLV : 1];
          col_loads(c, cv, KARGS);
          epilogue(z, r, c, v, cv, KARGS);
        } else epilogue(z, r, c, v, colv, KARGS);
      }
    }
#endif
  }
}
)KRN";

}  // namespace

const char* gemm_kernel_body() { return kGemmBody; }

// Source of the generated epilogue functions shared by the MatMul and Conv kernels:
//   col_loads()    operands addressed by the column alone (bias vectors, ...), loaded once per thread
//   epilogue()     one accumulator element: the block's successors of the anchor, then its store(s)
//   epilogue_vec() EPI_VEC consecutive columns of one row: the same expressions, with 16-byte
//                  vector loads/stores wherever an operand or destination is contiguous along the
//                  fastest column atom (defined when the column space allows it; EPI_VEC == 1 otherwise)
std::string gemm_epilogue_source(const LowerCtx& c, const std::vector<int>& batch, const std::vector<int>& rows,
                                 const std::vector<int>& cols, const std::map<int, int>& pslot, const std::string& kparams,
                                 int64_t GN, int row_bias_slot, int64_t GM) {
  const Graph& g = c.g;
  std::ostringstream k;
  // results larger than the L2 caches together (8 x 4 MB) plus some slack leave through non-temporal stores
  auto streamed = [&](int t) {
    const char* e = getenv("DNNF_STREAM_MB");      // (developer switch for A/B runs)
    return g.tensors[t].n() * dtype_bytes(g.tensors[t].dtype) >= ((int64_t)(e ? atoi(e) : 48) << 20);
  };
  std::set<int> need;
  {
    std::vector<int> stack;
    for (auto& s : c.stores) stack.push_back(s.value);
    while (!stack.empty()) {
      int n = stack.back();
      stack.pop_back();
      if (need.count(n)) continue;
      need.insert(n);
      for (int a : c.nodes[n].args) stack.push_back(a);
    }
  }
  std::map<int, std::string> col_override;
  for (int n : need) {
    const ENode& e = c.nodes[n];
    if (e.kind != ENode::LOAD || e.is_int || !e.addr.indirect.empty()) continue;
    Affine ea = c.resolved(e.addr);
    bool col_only = true;
    for (auto& kv : ea.stride)
      if (kv.second != 0 && std::find(cols.begin(), cols.end(), kv.first) == cols.end()) col_only = false;
    if (col_only) {
      int slot = (int)col_override.size();
      col_override[n] = "colv[" + std::to_string(slot) + "]";
    }
  }
  k << "#define NCOLV " << col_override.size() << "\n";
  k << "DEV void col_loads(idx_t cc, float* colv, " << kparams << ") {\n";
  decl_digits(k, c, cols, "cc", "  ", "qc");
  {
    int slot = 0;
    for (auto& kv : col_override) {
      const ENode& e = c.nodes[kv.first];
      k << "  colv[" << slot++ << "] = cvt_in(p" << pslot.at(e.tensor) << "[" << c.addr_expr(e.addr) << "]);\n";
    }
  }
  k << "}\n";
  k << "DEV void epilogue(idx_t z, idx_t r, idx_t cc, float anchor_v, const float* colv, " << kparams << ") {\n";
  decl_digits(k, c, batch, "z", "  ", "qz");
  decl_digits(k, c, rows, "r", "  ", "qr");
  decl_digits(k, c, cols, "cc", "  ", "qc");
  if (row_bias_slot >= 0) k << "  anchor_v += cvt_in(p" << row_bias_slot << "[r]);\n";
  // replication digits (a Resize behind the anchor): the successors and the stores run once per destination
  std::vector<int> reps;
  c.resolve(c.rep_atoms, reps);
  for (int ra : reps) k << "  for (idx_t a" << ra << " = 0; a" << ra << " < " << c.atom_extent[ra] << "; ++a" << ra << ")\n";
  k << "  {\n";
  {
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, "  ", &col_override);
    for (auto& s : c.stores) {
      std::string st = c.store_stmt(s, pslot, c.addr_expr(s.addr));
      if (s.preds.empty()) k << "  " << st << "\n";
      else k << "  if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
    }
  }
  k << "  }\n}\n";

  // ---- vector form: along the columns, else (destinations contiguous along the rows) along the rows,
  //      where the same generator runs with the two axes exchanged and the kernel reads its accumulator
  //      slab column-wise (EPI_T)
  int out_bytes = 4;
  for (auto& s : c.stores) out_bytes = std::min(out_bytes, dtype_bytes(g.tensors[s.tensor].dtype));
  bool stores_vectors = false;     // set by vector_form: some destination is written with vector stores
  auto vector_form = [&](const std::vector<int>& rows, const std::vector<int>& cols, int64_t GN, bool transposed) -> std::string {
  stores_vectors = false;
  if (!c.rep_atoms.empty()) return "";       // replicated results leave element by element
  std::ostringstream k;
  const int inner = cols.empty() ? -1 : cols.back(), outer = cols.size() >= 2 ? cols[cols.size() - 2] : -1;
  // A group of VE consecutive columns normally lies inside the fastest column atom.  It may also run
  // over the two fastest atoms (a 14-wide image row into the next row) when every address the epilogue
  // touches is linear in their combined index, i.e. stride(outer) = extent(inner) * stride(inner).
  auto linear_over_both = [&](const Affine& a0) {
    Affine a = c.resolved(a0);
    auto si = a.stride.find(inner), so = a.stride.find(outer);
    const int64_t vi = si == a.stride.end() ? 0 : si->second, vo = so == a.stride.end() ? 0 : so->second;
    return vo == vi * c.atom_extent[inner];
  };
  bool both_ok = outer >= 0;
  for (int n : need) if (c.nodes[n].kind == ENode::LOAD) both_ok = both_ok && c.nodes[n].addr.indirect.empty() && linear_over_both(c.nodes[n].addr);
  for (auto& s : c.stores) both_ok = both_ok && linear_over_both(s.addr);
  int VE = 0;
  bool cross = false;
  for (int ve = out_bytes == 2 ? 8 : 4; ve >= 4 && !VE && inner >= 0; ve /= 2) {
    if (GN % ve) continue;
    if (c.atom_extent[inner] % ve == 0) VE = ve;
    else if (both_ok && (c.atom_extent[inner] * c.atom_extent[outer]) % ve == 0) { VE = ve; cross = true; }
  }
  bool can = VE > 0;
  for (auto& s : c.stores) {
    can = can && dtype_bytes(g.tensors[s.tensor].dtype) == out_bytes;
    for (auto& pr : s.preds) {          // predicates must be uniform over a column group
      std::vector<int> r;
      c.resolve(pr.atoms, r);
      if (std::find(r.begin(), r.end(), inner) != r.end()) can = false;
      if (cross && std::find(r.begin(), r.end(), outer) != r.end()) can = false;
    }
  }
  if (!can) return "";
  auto contiguous = [&](const Affine& a0) {
    Affine a = c.resolved(a0);
    auto it = a.stride.find(inner);
    if (it == a.stride.end() || it->second != 1 || a.offset % VE != 0 || !a.indirect.empty()) return false;
    for (auto& kv : a.stride) if (kv.first != inner && !(cross && kv.first == outer) && kv.second % VE != 0) return false;
    return true;
  };
  for (auto& s : c.stores) stores_vectors = stores_vectors || contiguous(s.addr);
  if (transposed) {
    if (!stores_vectors) return "";   // worth it only if a destination really is contiguous along the rows
    k << "#define EPI_T 1\n";
  }
  k << "#define EPI_VEC " << VE << "\n";
  // r: index along the axis the group does not run along; cc: first index of the group along the other
  k << "DEV void epilogue_vec(idx_t z, idx_t r, idx_t cc, const float* accv, " << kparams << ") {\n";
  decl_digits(k, c, batch, "z", "  ", "qz");
  decl_digits(k, c, rows, "r", "  ", "qr");
  decl_digits(k, c, cols, "cc", "  ", "qc");      // atoms of the group's first column
  k << "  const idx_t inner0 = a" << inner << ";\n";
  std::map<int, std::string> ov;
  for (int n : need) {
    const ENode& e = c.nodes[n];
    if (e.kind != ENode::LOAD || e.is_int || !contiguous(e.addr)) continue;
    const Tensor& T = g.tensors[e.tensor];
    int lanes = dtype_bytes(T.dtype) == 2 ? 8 : 4;
    if (lanes < VE) continue;   // a 4-byte operand in an 8-wide group: leave it scalar
    k << "  typedef " << c.ctype(T.dtype) << " lv" << n << "_t __attribute__((ext_vector_type(" << VE << ")));\n";
    k << "  const lv" << n << "_t lv" << n << " = *(const lv" << n << "_t*)(p" << pslot.at(e.tensor) << " + (" << c.addr_expr(e.addr) << "));\n";
    ov[n] = "cvt_in(lv" + std::to_string(n) + "[u])";
  }
  std::vector<bool> vstore;
  for (size_t i = 0; i < c.stores.size(); i++) {
    vstore.push_back(contiguous(c.stores[i].addr));
    if (vstore[i]) {
      k << "  typedef " << c.ctype(g.tensors[c.stores[i].tensor].dtype) << " sv" << i << "_t __attribute__((ext_vector_type(" << VE << ")));\n";
      k << "  sv" << i << "_t sv" << i << ";\n";
    }
  }
  k << "#pragma unroll\n  for (int u = 0; u < " << VE << "; ++u) {\n";
  k << "    const idx_t a" << inner << " = inner0 + u;\n";
  k << "    float anchor_v = accv[u];\n";
  if (row_bias_slot >= 0) k << "    anchor_v += cvt_in(p" << row_bias_slot << "[" << (transposed ? "cc + u" : "r") << "]);\n";
  {
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, "    ", &ov);
    for (size_t i = 0; i < c.stores.size(); i++) {
      const Store& s = c.stores[i];
      if (vstore[i]) {
        k << "    { " << c.ctype(g.tensors[s.tensor].dtype) << " tmp; cvt_out(&tmp, " << c.vname(s.value) << "); sv" << i << "[u] = tmp; }\n";
      } else {
        std::string st = c.store_stmt(s, pslot, c.addr_expr(s.addr));
        if (s.preds.empty()) k << "    " << st << "\n";
        else k << "    if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
      }
    }
  }
  k << "  }\n";
  for (size_t i = 0; i < c.stores.size(); i++) {
    if (!vstore[i]) continue;
    const Store& s = c.stores[i];
    const std::string dst = "(sv" + std::to_string(i) + "_t*)(p" + std::to_string(pslot.at(s.tensor)) + " + (" + c.addr_expr(s.addr) + "))";
    std::string st = streamed(s.tensor) ? "dn_store_stream(" + dst + ", sv" + std::to_string(i) + ");" : "*" + dst + " = sv" + std::to_string(i) + ";";
    if (s.preds.empty()) k << "  " << st << "\n";
    else k << "  if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
  }
  k << "}\n";
  return k.str();
  };
  std::string vf = vector_form(rows, cols, GN, false);
  if ((vf.empty() || !stores_vectors) && GM > 0) {
    std::string vt = vector_form(cols, rows, GM, true);
    if (!vt.empty()) vf = vt;
  }
  if (vf.empty()) vf = "#define EPI_VEC 1\n";
  if (vf == "#define EPI_VEC 1\n" && c.rep_atoms.empty() && cols.size() == 1 && c.stores.size() == 1 && c.stores[0].preds.empty() &&
      (out_bytes == 2 || out_bytes == 4) && GN >= 64 && !getenv("DNNF_GEMM_NO_ROW_ALIGN")) {     // (developer switch for A/B runs)
    // No whole-vector form because the rows' starts are not 16-byte aligned (an odd row length): one result, contiguous
    // along a single column atom, can still leave as aligned vectors when every row is handled from its own first
    // aligned column on (the kernel shifts its accumulator slab row by row; see RA in the kernel body).
    const Store& s = c.stores[0];
    const int inner = cols[0], VE = 16 / out_bytes;
    Affine a = c.resolved(s.addr);
    auto it = a.stride.find(inner);
    if (it != a.stride.end() && it->second == 1 && a.indirect.empty() && dtype_bytes(g.tensors[s.tensor].dtype) == out_bytes) {
      std::ostringstream r;
      const std::string ct = c.ctype(g.tensors[s.tensor].dtype), ps = "p" + std::to_string(pslot.at(s.tensor));
      r << "#define EPI_RA " << VE << "\n";
      r << "DEV int epi_row_pad(idx_t z, idx_t r, idx_t cc, " << kparams << ") {\n";
      decl_digits(r, c, batch, "z", "  ", "qz");
      decl_digits(r, c, rows, "r", "  ", "qr");
      decl_digits(r, c, cols, "cc", "  ", "qc");
      r << "  return (int)(((unsigned long long)(" << ps << " + (" << c.addr_expr(s.addr) << ")) / " << out_bytes << ") % " << VE << ");\n}\n";
      r << "DEV void epilogue_ra(idx_t z, idx_t r, idx_t cc, const float* accv, " << kparams << ") {\n";
      decl_digits(r, c, batch, "z", "  ", "qz");
      decl_digits(r, c, rows, "r", "  ", "qr");
      decl_digits(r, c, cols, "cc", "  ", "qc");
      r << "  const idx_t inner0 = a" << inner << ";\n";
      r << "  typedef " << ct << " sv_t __attribute__((ext_vector_type(" << VE << ")));\n  sv_t sv;\n";
      r << "#pragma unroll\n  for (int u = 0; u < " << VE << "; ++u) {\n";
      r << "    const idx_t a" << inner << " = inner0 + u;\n    float anchor_v = accv[u];\n";
      if (row_bias_slot >= 0) r << "    anchor_v += cvt_in(p" << row_bias_slot << "[r]);\n";
      std::set<int> done;
      c.emit_values(r, {s.value}, done, pslot, "    ", nullptr);
      r << "    { " << ct << " tmp; cvt_out(&tmp, " << c.vname(s.value) << "); sv[u] = tmp; }\n  }\n";
      if (streamed(s.tensor)) r << "  dn_store_stream((sv_t*)(" << ps << " + (" << c.addr_expr(s.addr) << ")), sv);\n}\n";
      else r << "  *(sv_t*)(" << ps << " + (" << c.addr_expr(s.addr) << ")) = sv;\n}\n";
      vf += r.str();
    }
  }
  k << vf;
  return k.str();
}


MatmulFrame analyse_matmul(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  DNNF_CHECK(A.info->cls == OC_MATMUL, DNNF_UNSUPPORTED_OP, "only MatMul contractions have a kernel template");
  const Tensor& TA = g.tensors[A.in[0]];
  const Tensor& TB = g.tensors[A.in[1]];
  const Tensor& TC = g.tensors[A.out[0]];
  DNNF_CHECK(TA.dtype == TB.dtype && is_float(TA.dtype), DNNF_UNSUPPORTED_OP, "MatMul operands must share a float type");
  MatmulFrame f;
  f.dtype = TA.dtype;
  size_t ro = TC.dims.size();
  TIdx oi = c.fresh_index(TC.dims);
  int64_t K = TA.dims.back();
  DNNF_CHECK(K >= 1, DNNF_UNSUPPORTED_OP, "empty contraction");
  f.K = K;
  int katom = c.new_atom(K);
  auto operand_idx = [&](const Tensor& T, bool is_a) {
    TIdx ix(T.dims.size());
    size_t nb = T.dims.size() - 2, shift = (ro - 2) - nb;
    for (size_t d = 0; d < nb; d++)
      if (T.dims[d] != 1) ix[d] = oi[d + shift];
    if (is_a) { ix[nb] = oi[ro - 2]; if (K > 1) ix[nb + 1].atoms = {katom}; }
    else { if (K > 1) ix[nb].atoms = {katom}; ix[nb + 1] = oi[ro - 1]; }
    return ix;
  };
  TIdx ai = operand_idx(TA, true), bi = operand_idx(TB, false);
  c.tidx[c.anchor_out] = oi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.allow_replication = true;
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the contraction");
  c.collect_stores(eout);
  int an = c.value(A.in[0], ai), bn = c.value(A.in[1], bi);
  DNNF_CHECK(c.nodes[an].kind == ENode::LOAD && c.nodes[bn].kind == ENode::LOAD && c.nodes[an].addr.indirect.empty() &&
                 c.nodes[bn].addr.indirect.empty(),
             DNNF_UNSUPPORTED_OP, "arithmetic in front of a contraction operand has no kernel template");
  f.ta = c.nodes[an].tensor;
  f.tb = c.nodes[bn].tensor;
  DNNF_CHECK(g.tensors[f.ta].dtype == TA.dtype && g.tensors[f.tb].dtype == TA.dtype, DNNF_UNSUPPORTED_OP, "operand dtype changes in prologue");
  f.aa = c.resolved(c.nodes[an].addr);
  f.ab = c.resolved(c.nodes[bn].addr);
  Affine ac = c.resolved(c.affine(TC, oi));

  // classify the output atoms
  c.resolve({katom}, f.katoms);
  std::vector<int> fin = c.final_atoms();
  for (int at : fin) {
    if (std::find(f.katoms.begin(), f.katoms.end(), at) != f.katoms.end()) continue;
    if (!stride_of(ac, at)) continue;   // not an output atom (cannot happen for a MatMul)
    bool ia = stride_of(f.aa, at) != 0, ib = stride_of(f.ab, at) != 0;
    // an atom of the M (N) axis belongs to the rows (columns) even if its operand is broadcast
    if (ia && !ib) f.rows.push_back(at);
    else if (ib && !ia) f.cols.push_back(at);
    else f.batch.push_back(at);
  }
  // atoms of the M and N axes that neither operand strides over (extent-1 operands) stay where the output has them
  auto by_c = [&](int x, int y) { return stride_of(ac, x) > stride_of(ac, y); };
  std::sort(f.rows.begin(), f.rows.end(), by_c);
  std::sort(f.cols.begin(), f.cols.end(), by_c);
  std::sort(f.batch.begin(), f.batch.end(), by_c);
  f.GM = c.extent_of(f.rows);
  f.GN = c.extent_of(f.cols);
  f.GZ = c.extent_of(f.batch);

  const int eb = dtype_bytes(TA.dtype), VEC = eb == 2 ? 8 : 4;
  auto mode_of = [&](const Affine& a, const std::vector<int>& other, int64_t other_extent) {
    // 0 direct (K-contiguous), 1 transpose (contiguous along the other axis), 2 scalar
    auto aligned = [&](int skip) {
      if (a.offset % VEC) return false;
      for (auto& kv : a.stride) if (kv.first != skip && kv.second % VEC) return false;
      return true;
    };
    if (!f.katoms.empty()) {
      int kin = f.katoms.back();
      if (stride_of(a, kin) == 1 && c.atom_extent[kin] % VEC == 0 && aligned(kin)) return 0;
    } else if (K == 1) return 2;
    if (!other.empty()) {
      int oin = -1;
      for (int at : other) if (stride_of(a, at) == 1) oin = at;
      if (oin >= 0 && oin == other.back() && c.atom_extent[oin] % VEC == 0 && aligned(oin) && other_extent % VEC == 0) return 1;
    }
    return 2;
  };
  f.amode = mode_of(f.aa, f.rows, f.GM);
  f.bmode = mode_of(f.ab, f.cols, f.GN);
  return f;
}

Lowered lower_gemm(LowerCtx& c, LowerCtx* norm, int norm_in, bool norm_in_stored) {
  const Graph& g = c.g;
  MatmulFrame fr = analyse_matmul(c);
  const Tensor& TA = g.tensors[g.ops[c.anchor_op].in[0]];
  const int64_t K = fr.K, GM = fr.GM, GN = fr.GN, GZ = fr.GZ;
  const int ta = fr.ta, tb = fr.tb;
  const Affine& aa = fr.aa;
  const Affine& ab = fr.ab;
  const std::vector<int>&katoms = fr.katoms, &rows = fr.rows, &cols = fr.cols, &batch = fr.batch;
  const std::vector<int>&rows_a = rows, &cols_b = cols;
  const int eb = dtype_bytes(TA.dtype);
  int amode = fr.amode, bmode = fr.bmode;

  // ---- tile configuration
  struct Cfg { int BM, BN, BK, WM, WN, WK, NBUF, PF, DMA = 0; };
  auto nblocks = [&](int bm, int bn) { return ((GM + bm - 1) / bm) * ((GN + bn - 1) / bn) * GZ; };
  const int BK0 = eb == 2 ? (K <= 32 ? 32 : 64) : 16;
  std::vector<Cfg> cands;
  for (auto t : {std::pair<int, int>{128, 128}, {128, 64}, {64, 128}, {64, 64}}) cands.push_back({t.first, t.second, BK0, 2, 2, 1, 1, 2});
  cands.push_back({64, 64, BK0, 2, 2, 1, 2, 3});
  // deeper prefetch for the products that stream one large operand from HBM (attention probabilities, scores):
  // their speed is the number of bytes a compute unit keeps in flight
  cands.push_back({128, 64, BK0, 2, 2, 1, 2, 4});
  cands.push_back({64, 64, BK0, 2, 2, 1, 2, 4});
  // eight wavefronts on a larger tile: fewer LDS stores per MFMA (stores run at half the rate of loads)
  if (eb == 2 && BK0 == 64) {
    cands.push_back({256, 128, BK0, 4, 2, 1, 1, 2});
    cands.push_back({256, 256, BK0, 4, 2, 1, 2, 2});
    // eight wavefronts on a 128x128 tile (two rows of four, 64x32 results each): twice the fragment reads per MFMA of
    // the four-wavefront form, but two workgroups of eight per compute unit keep four wavefronts on every SIMD, and
    // short products (K of 768: a dozen K tiles between a tile's first load and its epilogue) are bound by latency,
    // not by LDS - measured 15 % faster than any other configuration on the M = 4096 layer products of config 5
    cands.push_back({128, 128, BK0, 2, 4, 1, 2, 2});
    cands.push_back({128, 128, BK0, 2, 4, 1, 1, 2});
    // and sixteen (the largest workgroup the chip takes: four wavefronts per SIMD from one workgroup) on 256x256 and
    // 128x128: 64x64 / 32x32 results per wavefront.  19 % faster than the eight-wavefront 256x256 tile on the
    // vocabulary product of config 5
    cands.push_back({256, 256, BK0, 4, 4, 1, 2, 2});
    cands.push_back({128, 128, BK0, 4, 4, 1, 2, 2});
  }
  // both operands contiguous along K and K a whole number of tiles: tiles loaded straight into LDS
  const bool dma_ok = eb == 2 && amode == 0 && bmode == 0 && K % 64 == 0 && !getenv("DNNF_GEMM_NO_DMA");   // (developer switch for A/B runs)
  if (dma_ok) {
    cands.push_back({64, 64, 64, 2, 2, 1, 2, 1, 1});
    // larger tiles on the same loop: 128 KB / 64 KB of LDS for the two buffers, eight wavefronts on the 256x256
    // tile (two per SIMD, 64x128 results each), four on 128x128
    cands.push_back({256, 256, 64, 4, 2, 1, 2, 1, 1});
    cands.push_back({128, 128, 64, 2, 2, 1, 2, 1, 1});
    // the same loop with eight wavefronts per workgroup
    cands.push_back({128, 128, 64, 2, 4, 1, 2, 1, 1});
    cands.push_back({64, 128, 64, 2, 4, 1, 2, 1, 1});
    cands.push_back({128, 64, 64, 4, 2, 1, 2, 1, 1});
    cands.push_back({256, 256, 64, 4, 4, 1, 2, 1, 1});
  }
  // Default choice: a cost model in cycles per CU.  A K tile costs the larger of its MFMA time and its
  // LDS time (16-byte fragment reads at 128 B/clk, stores at 64 B/clk) plus a fixed barrier/latency
  // share; tiles are dealt to 256 CUs, and partly filled rounds count in full.
  auto cost = [&](const Cfg& f) {
    const double tm = f.BM / f.WM / 32.0, tn = f.BN / f.WN / 32.0, steps = f.BK / 16.0;
    const double mfma = tm * tn * steps * (eb == 2 ? 32.0 : 512.0) * (f.WM * f.WN / 4.0);   // wavefronts share 4 SIMDs
    const double lds_rd = f.WM * f.WN * (tm + tn) * steps * 8.0;
    const double lds_wr = (f.BM + f.BN) * f.BK * eb / 64.0;
    const double nkt = (double)((K + f.BK - 1) / f.BK);
    const double per_tile = nkt * (std::max(mfma, lds_rd + lds_wr) + 120.0) + f.BM * f.BN / 16.0 + 1500.0;
    const double rounds = std::ceil((double)nblocks(f.BM, f.BN) / 256.0);
    return rounds * per_tile * (f.DMA ? 0.9 : 1.0);
  };
  int pick = 0;
  if (c.opts.force_variant >= 100) {
    DNNF_CHECK(c.opts.force_variant - 100 < (int)cands.size(), DNNF_UNSUPPORTED_OP, "no such GEMM tile variant");
    pick = c.opts.force_variant - 100;
  } else {
    for (size_t i = 1; i < cands.size(); i++)
      if (cost(cands[i]) < cost(cands[pick])) pick = (int)i;
  }
  Cfg f = cands[pick];
  // a problem too small to occupy the chip with 64x64 tiles: 32x32 tiles, the four wavefronts of a
  // workgroup splitting K between them
  if (c.opts.force_variant < 100 && nblocks(64, 64) < 192 && K >= 8 * BK0) f = {32, 32, BK0, 1, 1, 4, 1, 2};
  int BM = f.BM, BN = f.BN, BK = f.BK, WAVES_M = f.WM, WAVES_N = f.WN, WAVES_K = f.WK, NBUF = f.NBUF, PF = f.PF, DMA = f.DMA;
  // developer override for tuning runs: DNNF_GEMM_TILE=BM,BN,BK,WAVES_M,WAVES_N,NBUF[,PF[,DMA[,MIN_N]]]
  if (const char* ov = getenv("DNNF_GEMM_TILE")) {
    // (a ninth and a tenth field restrict the override to unbatched products of at least / at most that many columns)
    int v[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    if (sscanf(ov, "%d,%d,%d,%d,%d,%d,%d,%d,%d,%d", v, v + 1, v + 2, v + 3, v + 4, v + 5, v + 6, v + 7, v + 8, v + 9) >= 6 && GN >= v[8] && (v[9] == 0 || (GN <= v[9] && GZ == 1)) &&
        v[3] > 0 && v[4] > 0 && 16 % (v[3] * v[4]) == 0 &&
        v[0] % (32 * v[3]) == 0 && v[1] % (32 * v[4]) == 0 && v[2] % (eb == 2 ? 16 : 4) == 0 && (v[5] == 1 || v[5] == 2 || (v[7] == 1 && v[5] <= 4 && v[5] >= 1))) {
      BM = v[0]; BN = v[1]; BK = v[2]; WAVES_M = v[3]; WAVES_N = v[4]; NBUF = v[5]; WAVES_K = std::max(1, 4 / (v[3] * v[4]));
      if (v[6] >= 1 && v[6] <= 4) PF = v[6];
      DMA = v[7] == 1 && dma_ok && BK == 64 && NBUF >= 2 && WAVES_K == 1;
    }
  }
  int norm_value = -1;        // expression node of the value the normalisation reads
  if (norm) {
    // eight wavefronts side by side on 32 whole rows of the product
    DNNF_CHECK(GN <= 768, DNNF_UNSUPPORTED_OP, "normalised rows longer than 768 columns do not fit one workgroup's tile");
    BM = 32; BN = (int)((GN + 255) / 256 * 256); BK = BK0; WAVES_M = 1; WAVES_N = 8; WAVES_K = 1; NBUF = 1; PF = 1; DMA = 0;
    // the normalised tensor is the product's own index space: batch and rows lead, the columns are its last axis
    const TIdx& xi = c.tidx.at(norm_in);
    std::vector<int> last, lead, want = batch;
    want.insert(want.end(), rows.begin(), rows.end());
    c.resolve(xi.back().atoms, last);
    DNNF_CHECK(last == cols && xi.back().offset == 0 && xi.back().indirect < 0, DNNF_UNSUPPORTED_OP, "the normalised axis is not the product's column axis");
    for (size_t d = 0; d + 1 < xi.size(); d++) {
      DNNF_CHECK(xi[d].offset == 0 && xi[d].indirect < 0, DNNF_UNSUPPORTED_OP, "sliced rows in front of the normalisation");
      c.resolve(xi[d].atoms, lead);
    }
    DNNF_CHECK(lead == want, DNNF_UNSUPPORTED_OP, "operators in front of the normalisation permute the product's rows");
    DNNF_CHECK(c.rep_atoms.empty(), DNNF_UNSUPPORTED_OP, "replicated results in front of a normalisation");
    for (size_t i = 0; i < c.stores.size(); i++)
      if (c.stores[i].tensor == norm_in) {
        DNNF_CHECK(c.stores[i].preds.empty(), DNNF_UNSUPPORTED_OP, "the normalised tensor is only partly written");
        norm_value = c.stores[i].value;
        if (!norm_in_stored) { c.stores.erase(c.stores.begin() + (long)i); break; }
      }
    DNNF_CHECK(norm_value >= 0, DNNF_UNSUPPORTED_OP, "the normalised tensor is not produced by the product's part of the block");
  }
  // a wavefront's load instruction fills 64 whole 16-byte slots of the tile: no partly used pass
  if (DMA) DNNF_CHECK((BM * BK / 8) % (64 * WAVES_M * WAVES_N) == 0 && (BN * BK / 8) % (64 * WAVES_M * WAVES_N) == 0, DNNF_UNSUPPORTED_OP, "tile does not divide into whole load passes");

  // parameters: A, B, epilogue loads, outputs
  std::vector<int> params = {ta, tb};
  std::map<int, int> pslot;
  std::set<int> written;
  {
    // epilogue operands get their own parameter slots even if they alias A or B
    auto collect = [&](const LowerCtx& cx, std::vector<int> stack) {
      std::set<int> need;
      while (!stack.empty()) {
        int n = stack.back();
        stack.pop_back();
        if (need.count(n)) continue;
        need.insert(n);
        for (int a : cx.nodes[n].args) stack.push_back(a);
        if (cx.nodes[n].kind == ENode::LOAD) for (auto& p : cx.nodes[n].addr.indirect) stack.push_back(p.first);
      }
      for (int n : need)
        if (cx.nodes[n].kind == ENode::LOAD && !pslot.count(cx.nodes[n].tensor)) {
          pslot[cx.nodes[n].tensor] = (int)params.size();
          params.push_back(cx.nodes[n].tensor);
        }
    };
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    if (norm_value >= 0) roots.push_back(norm_value);
    collect(c, roots);
    if (norm) {
      roots.clear();
      for (auto& s : norm->stores) roots.push_back(s.value);
      collect(*norm, roots);
      DNNF_CHECK(!pslot.count(norm_in) || norm_in_stored, DNNF_UNSUPPORTED_OP, "the normalised tensor is read from memory inside its own block");
    }
  }
  size_t n_in = params.size();
  auto add_stores = [&](const LowerCtx& cx) {
    for (auto& s : cx.stores) {
      DNNF_CHECK(!pslot.count(s.tensor) && s.tensor != ta && s.tensor != tb, DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
      pslot[s.tensor] = (int)params.size();
      params.push_back(s.tensor);
      written.insert(s.tensor);
    }
  };
  add_stores(c);
  if (norm) add_stores(*norm);
  const bool wide = [&] {
    for (int t : params) if (g.tensors[t].n() >= (int64_t)1 << 31) return true;
    return false;
  }();

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "typedef " << c.ctype(TA.dtype) << " elem_t;\n";
  k << "#define ELEM_BYTES " << eb << "\n#define BM " << BM << "\n#define BN " << BN << "\n#define BK " << BK << "\n";
  k << "#define GM " << GM << "\n#define GN " << GN << "\n#define GK " << K << "\n";
  k << "#define WAVES_M " << WAVES_M << "\n#define WAVES_N " << WAVES_N << "\n#define WAVES_K " << WAVES_K << "\n#define NBUF " << NBUF << "\n#define PF " << PF << "\n";
  k << "#define A_MODE " << amode << "\n#define B_MODE " << bmode << "\n#define PA p0\n#define PB p1\n";
  if (DMA) k << "#define DMA 1\n";
  {
    // a weight operand of up to 16 MB that the block reads whole (dense, no batch): touched by every XCD up front
    const Tensor& TBt = g.tensors[tb];
    const int64_t wbytes = TBt.n() * dtype_bytes(TBt.dtype);
    if (!norm && GZ == 1 && (TBt.kind == DNNF_WEIGHT || TBt.weight_only) && wbytes >= (256 << 10) && wbytes <= ((int64_t)16 << 20) &&
        wbytes == GN * K * eb && !getenv("DNNF_NO_WEIGHT_PREFETCH"))      // (developer switch for A/B runs)
      k << "#define W_PREFETCH_LINES " << wbytes / 128 << "\n#define W_PREFETCH_PTR p1\n";
  }
  if (TA.dtype == DNNF_F16) k << "typedef f16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16\n";
  else if (TA.dtype == DNNF_BF16) k << "typedef bf16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16\n";
  k << offset_fn(c, "offA_row", rows_a, aa) << offset_fn(c, "offA_k", katoms, aa) << offset_fn(c, "offA_batch", batch, aa);
  k << offset_fn(c, "offB_col", cols_b, ab) << offset_fn(c, "offB_k", katoms, ab) << offset_fn(c, "offB_batch", batch, ab);
  // epilogue
  std::string kparams = c.param_list(params, written), kargs;
  for (size_t i = 0; i < params.size(); i++) kargs += (i ? ", p" : "p") + std::to_string(i);
  if (!norm) k << gemm_epilogue_source(c, batch, rows, cols, pslot, kparams, GN, -1, GM);
  else {
    const Op& NM = g.ops[norm->anchor_op];
    k << "#define EPI_ROWNORM 1\n#define EPI_VEC 1\n#define NCOLV 0\n#define NORM_EPS " << (float)NM.f("epsilon", 1e-5) << "f\n";
    k << "DEV void col_loads(idx_t cc, float* colv, " << kparams << ") {}\n";
    k << "DEV void epilogue(idx_t z, idx_t r, idx_t cc, float anchor_v, const float* colv, " << kparams << ") {}\n";
    // the product's part: its operators and stores, and the value the normalisation reads (as it would read it back
    // from memory: rounded to the tensor's storage type)
    k << "DEV float gn_value(idx_t z, idx_t r, idx_t cc, float anchor_v, " << kparams << ") {\n";
    decl_digits(k, c, batch, "z", "  ", "qz");
    decl_digits(k, c, rows, "r", "  ", "qr");
    decl_digits(k, c, cols, "cc", "  ", "qc");
    {
      std::set<int> done;
      std::vector<int> roots = {norm_value};
      for (auto& s : c.stores) roots.push_back(s.value);
      c.emit_values(k, roots, done, pslot, "  ");
      for (auto& s : c.stores) k << "  " << c.store_stmt(s, pslot, c.addr_expr(s.addr)) << "\n";
      for (auto& s : c.stores) DNNF_CHECK(s.preds.empty(), DNNF_UNSUPPORTED_OP, "predicated store in front of a normalisation");
    }
    k << "  " << c.ctype(g.tensors[norm_in].dtype) << " t_; cvt_out(&t_, " << c.vname(norm_value) << ");\n  return cvt_in(t_);\n}\n";
    // the normalisation's part: row = position among all rows of the normalised tensor, cc = column
    std::vector<int> nrow, ncol;
    {
      const TIdx& yi = norm->tidx.at(norm->anchor_out);
      for (size_t d = 0; d + 1 < yi.size(); d++) norm->resolve(yi[d].atoms, nrow);
      norm->resolve(yi.back().atoms, ncol);
    }
    k << "DEV void gn_store(idx_t row, idx_t cc, float anchor_v, " << kparams << ") {\n";
    decl_digits(k, *norm, nrow, "row", "  ", "qr");
    decl_digits(k, *norm, ncol, "cc", "  ", "qc");
    {
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s : norm->stores) roots.push_back(s.value);
      norm->emit_values(k, roots, done, pslot, "  ");
      for (auto& s : norm->stores) {
        std::string st = norm->store_stmt(s, pslot, norm->addr_expr(s.addr));
        if (s.preds.empty()) k << "  " << st << "\n";
        else k << "  if (" << norm->pred_expr(s.preds) << ") { " << st << " }\n";
      }
    }
    k << "}\n";
  }
  k << "#define KPARAMS " << kparams << "\n#define KARGS " << kargs << "\n";
  k << kGemmBody;

  Lowered Lw;
  Lw.family = FAM_GEMM;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch Kn;
  Kn.params = params;
  Kn.grid[0] = (unsigned)nblocks(BM, BN);
  Kn.block[0] = 64 * WAVES_M * WAVES_N * WAVES_K;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_gemm", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  Lw.variant = "mfma_" + std::to_string(BM) + "x" + std::to_string(BN) + "x" + std::to_string(BK) + "_a" + std::to_string(amode) + "b" + std::to_string(bmode) +
               (WAVES_M * WAVES_N * WAVES_K > 4 ? "_w" + std::to_string(WAVES_M * WAVES_N * WAVES_K) : std::string()) + (DMA ? (NBUF > 2 ? "_dma" + std::to_string(NBUF) : std::string("_dma")) : std::string()) + (norm ? "_rownorm" : "");
  return Lw;
}

// MatMul -> One-to-One operators -> normalisation of the last axis (LayerNorm statistics) -> One-to-One operators as
// one block.  The mapping-type table keeps a Many-to-Many operator behind another one apart (Sec. 3.2, red); this
// form exists because a tile that holds whole rows of the product has the normalisation's input on chip.  The block
// is split at the normalisation: what its input depends on is lowered as a MatMul block whose "result" is the
// normalised tensor, the normalisation and what follows it as a second expression over the same rows and columns.
Lowered lower_gemm_norm(const Graph& g, const Block& b, const LowerOpts& o) {
  int nm = -1, mm = -1;
  for (int oi : b.ops) {
    if (g.ops[oi].info->cls == OC_NORMALIZE) { DNNF_CHECK(nm < 0, DNNF_UNSUPPORTED_OP, "two normalisations in one block"); nm = oi; }
    if (g.ops[oi].info->cls == OC_MATMUL) { DNNF_CHECK(mm < 0, DNNF_UNSUPPORTED_OP, "two contractions in one block"); mm = oi; }
  }
  DNNF_CHECK(nm >= 0 && mm >= 0, DNNF_UNSUPPORTED_OP, "not a MatMul - normalisation block");
  const Op& NM = g.ops[nm];
  DNNF_CHECK(NM.kind == "Normalize", DNNF_UNSUPPORTED_OP, "only the normalisation of the last axis joins a MatMul block");
  const int X = NM.in[0];
  // operators that depend on the normalisation's result form the second part
  std::set<int> in_block(b.ops.begin(), b.ops.end()), after;
  {
    std::vector<int> stack = {nm};
    while (!stack.empty()) {
      int op = stack.back();
      stack.pop_back();
      if (after.count(op)) continue;
      after.insert(op);
      for (int t : g.ops[op].out)
        for (int cns : g.tensors[t].consumers) if (in_block.count(cns)) stack.push_back(cns);
    }
  }
  DNNF_CHECK(!after.count(mm), DNNF_UNSUPPORTED_OP, "the contraction must come before the normalisation");
  Block bg, bn;
  for (int oi : b.ops) (after.count(oi) ? bn : bg).ops.push_back(oi);
  bg.fused_type = bn.fused_type = DNNF_MANY_TO_MANY;
  for (int oi : bn.ops) {
    const OpClass cl = g.ops[oi].info->cls;
    DNNF_CHECK(oi == nm || (cl != OC_REDUCE && cl != OC_SOFTMAX && cl != OC_NORMALIZE && cl != OC_GAP && cl != OC_CONV && cl != OC_MATMUL &&
                            cl != OC_POOL && cl != OC_SCAN && cl != OC_CONCAT && cl != OC_CONVT && cl != OC_GEMM),
               DNNF_UNSUPPORTED_OP, "a further Many-to-Many operator behind the normalisation");
  }
  std::vector<int> ein, eout, removed;
  block_io(g, b, ein, eout, removed);
  const bool x_stored = std::find(eout.begin(), eout.end(), X) != eout.end();
  DNNF_CHECK(x_stored || std::find(removed.begin(), removed.end(), X) != removed.end(), DNNF_UNSUPPORTED_OP,
             "the normalised tensor is not computed inside the block");

  LowerCtx cg(g, bg, o), cn(g, bn, o);
  cg.anchor_op = mm;
  cg.anchor_out = g.ops[mm].out[0];
  cn.anchor_op = nm;
  cn.anchor_out = NM.out[0];
  // the normalisation's part over the index space of its input (as the row-reduction template sets it up)
  cn.tidx[cn.anchor_out] = cn.fresh_index(g.tensors[X].dims);
  {
    std::vector<int> ein_n, eout_n, rem_n;
    block_io(g, bn, ein_n, eout_n, rem_n);
    cn.forward_all();
    for (int t : eout_n)
      DNNF_CHECK(cn.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the normalisation");
    cn.collect_stores(eout_n);
    DNNF_CHECK(cn.rep_atoms.empty(), DNNF_UNSUPPORTED_OP, "replicated results behind a normalisation");
  }
  return lower_gemm(cg, &cn, X, x_stored);
}

}  // namespace dnnf
