// Streaming-softmax attention block: MatMul -> One-to-One operators -> Softmax -> MatMul (+ the
// second MatMul's successors) in one kernel, so that the score matrix never reaches memory.
//
// The mapping-type analysis marks Many-to-Many followed by Many-to-Many red (Sec. 3.2), so the
// paper's planner never forms this block; it is offered as an extension behind a plan option.  What
// makes it legal is an algebraic property of Softmax the table does not look at: the row maximum and
// row sum can be carried along while the keys are visited tile by tile, rescaling the partial result.
//
// Kernel shape (gfx950): 256 threads = 4 wavefronts, each owning 32 query rows of a 128-row tile.
// Per 64-key step a wavefront computes S^T = K_tile . Q^T with 32x32x16 MFMAs (A = keys from LDS, B =
// its queries, resident in registers).  In the accumulator layout a lane then holds one query and,
// in its registers, keys - so the softmax statistics are reductions over a lane's own registers plus
// one exchange between the two half-waves.  The probabilities, rounded to the operand type, are
// already laid out as the B fragments of O^T = V^T . P^T: registers [8s, 8s+8) of a score tile are
// the lane's eight K slots of MFMA step s, provided the V tile is stored in LDS with its keys in
// the matching slot order (within each group of 16 keys the quads are stored as 0, 2, 1, 3).
// The generated score function applies the block's One-to-One operators (scaling, masks) to four
// consecutive keys at a time; the generated epilogue is the GEMM template's (LDS-staged, vector stores).
#include <algorithm>
#include <set>
#include <sstream>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {

const char* kAttnBody = R"KRN(
#define BQ 128                         // queries per workgroup: 4 wavefronts x 32
#define BJ 64                          // keys per step
#define LDK (DH + 8)                   // row pitch of the key tile [key][d]
#define LDV (BJ + 8)                   // row pitch of the value tile [dv][key slot]
#define TD (DV / 32)
#define KS (DH / 16)
#define CLD (DV + 4)                   // row pitch of the fp32 output slab
#define KV_BYTES (2 * 2 * (BJ * LDK + DV * LDV))
#define CS_BYTES (4 * BQ * CLD)
#define LOG2E 1.44269504f
#define K_VECS ((BJ * DH / 8 + 255) / 256)
#define V_VECS ((BJ * DV / 8 + 255) / 256)
#define K_SUB ((BJ * DH / 64 + 255) / 256)
#define V_SUB ((BJ * DV / 16 + 255) / 256)   // sub-blocks of 8 keys x 2 channels

extern "C" __global__ __launch_bounds__(256) void KNAME(KPARAMS) {
  __shared__ __attribute__((aligned(16))) char smem[KV_BYTES > CS_BYTES ? KV_BYTES : CS_BYTES];
  typedef elem_t (*ktile_t)[BJ][LDK];
  typedef elem_t (*vtile_t)[DV][LDV];
  const ktile_t Ks = (ktile_t)smem;
  const vtile_t Vt = (vtile_t)(smem + 2 * 2 * BJ * LDK);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, l31 = lane & 31;
  const idx_t qtiles = (SQ + BQ - 1) / BQ;
  const idx_t z = blockIdx.x / qtiles, q0 = (blockIdx.x % qtiles) * BQ;
  const elem_t* __restrict__ Qb = PQ + offQ_batch(z);
  const elem_t* __restrict__ Kb = PK + offK_batch(z);
  const elem_t* __restrict__ Vb = PV + offV_batch(z);

  // this lane's query row (clamped at the edge: such rows are computed and never stored)
  const idx_t qi = q0 + wave * 32 + l31, qic = qi < SQ ? qi : (idx_t)(SQ - 1);
  frag_t rq[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) rq[ks] = __builtin_bit_cast(frag_t, *(const u16x8*)(Qb + offQ_row(qic) + offQ_k(ks * 16 + h * 8)));

  f32x16 oacc[TD];
#pragma unroll
  for (int t = 0; t < TD; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[t][e] = 0.0f;
  float m_run = -__builtin_inff(), l_run = 0.0f;

  // ---- key / value tile loaders: global -> registers -> LDS
#if K_MODE == 0
  u16x8 rk[K_VECS];
#else
  u16x8 rk[K_SUB][8];
#endif
#if V_MODE == 0
  u16x8 rv[V_VECS];
#else
  u16x2 rv[V_SUB][8];
#endif
#define KEY(j) ((SK % BJ == 0) ? (idx_t)(j) : ((j) < SK ? (idx_t)(j) : (idx_t)(SK - 1)))
#define KEY4(j) ((SK % BJ == 0) ? (idx_t)(j) : ((j) < SK ? (idx_t)(j) : (idx_t)(SK - 4)))   // start of a group of 4 keys
  auto gload = [&](const idx_t j0) {
#if K_MODE == 0
    // keys stored [key][d], d contiguous: one 16-byte vector per (key, d-octet)
#pragma unroll
    for (int i = 0; i < K_VECS; ++i) {
      const int v = (BJ * DH / 8 % 256 == 0 || tid + i * 256 < BJ * DH / 8) ? tid + i * 256 : 0;
      const int j = v / (DH / 8), dk = (v % (DH / 8)) * 8;
      rk[i] = *(const u16x8*)(Kb + offK_col(KEY(j0 + j)) + offK_k(dk));
    }
#else
    // keys stored [d][key], key contiguous: a thread owns an 8 x 8 sub-block and transposes it
#pragma unroll
    for (int i = 0; i < K_SUB; ++i) {
      const int s = (BJ * DH / 64 % 256 == 0 || tid + i * 256 < BJ * DH / 64) ? tid + i * 256 : 0;
      const int jb = (s % (BJ / 8)) * 8, db = (s / (BJ / 8)) * 8;
      const idx_t co = offK_col(KEY(j0 + jb) / 8 * 8);
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) rk[i][jj] = *(const u16x8*)(Kb + co + offK_k(db + jj));
    }
#endif
#if V_MODE == 0
    // values stored [dv][key], key contiguous
#pragma unroll
    for (int i = 0; i < V_VECS; ++i) {
      const int v = (BJ * DV / 8 % 256 == 0 || tid + i * 256 < BJ * DV / 8) ? tid + i * 256 : 0;
      const int dv = v / (BJ / 8), jb = (v % (BJ / 8)) * 8;
      rv[i] = *(const u16x8*)(Vb + offV_col(dv) + offV_k(KEY(j0 + jb) / 8 * 8));
    }
#else
    // values stored [key][dv], dv contiguous: a thread owns 8 keys x 2 channels (every thread takes part in the
    // transposition; neighbouring threads read neighbouring channel pairs of the same keys)
#pragma unroll
    for (int i = 0; i < V_SUB; ++i) {
      const int s = (BJ * DV / 16 % 256 == 0 || tid + i * 256 < BJ * DV / 16) ? tid + i * 256 : 0;
      const int db = (s % (DV / 2)) * 2, jb = (s / (DV / 2)) * 8;
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) rv[i][jj] = *(const u16x2*)(Vb + offV_k(KEY(j0 + jb + jj)) + offV_col(db));
    }
#endif
  };
  // eight consecutive keys starting at a multiple of 8 land in two quads of their group of 16
  auto put_v = [&](const int buf, const int dv, const int jb, const u16x8 o) {
    const int base = (jb / 16) * 16 + ((jb % 16) / 8) * 4;
    *(u16x4*)&Vt[buf][dv][base] = (u16x4){o[0], o[1], o[2], o[3]};
    *(u16x4*)&Vt[buf][dv][base + 8] = (u16x4){o[4], o[5], o[6], o[7]};
  };
  auto lstore = [&](const int buf) {
#if K_MODE == 0
#pragma unroll
    for (int i = 0; i < K_VECS; ++i) {
      const int v = tid + i * 256, j = v / (DH / 8), dk = (v % (DH / 8)) * 8;
      if (BJ * DH / 8 % 256 == 0 || v < BJ * DH / 8) *(u16x8*)&Ks[buf][j][dk] = rk[i];
    }
#else
#pragma unroll
    for (int i = 0; i < K_SUB; ++i) {
      const int s = tid + i * 256, jb = (s % (BJ / 8)) * 8, db = (s / (BJ / 8)) * 8;
      if (BJ * DH / 64 % 256 == 0 || s < BJ * DH / 64) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          u16x8 o;
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) o[jj] = rk[i][jj][r];
          *(u16x8*)&Ks[buf][jb + r][db] = o;
        }
      }
    }
#endif
#if V_MODE == 0
#pragma unroll
    for (int i = 0; i < V_VECS; ++i) {
      const int v = tid + i * 256, dv = v / (BJ / 8), jb = (v % (BJ / 8)) * 8;
      if (BJ * DV / 8 % 256 == 0 || v < BJ * DV / 8) put_v(buf, dv, jb, rv[i]);
    }
#else
#pragma unroll
    for (int i = 0; i < V_SUB; ++i) {
      const int s = tid + i * 256, db = (s % (DV / 2)) * 2, jb = (s / (DV / 2)) * 8;
      if (BJ * DV / 16 % 256 == 0 || s < BJ * DV / 16) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          u16x8 o;
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) o[jj] = rv[i][jj][r];
          put_v(buf, db + r, jb, o);
        }
      }
    }
#endif
  };

  const int nj = (SK + BJ - 1) / BJ;
  // operands of the score operators (masks) for one key tile: 2 x 4 groups of four keys per lane
  sload_t sl[2][4], sl_next[2][4];
  auto sload = [&](sload_t (&dst)[2][4], const idx_t j0) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) dst[t][q] = score_load(z, qic, KEY4(j0 + t * 32 + q * 8 + h * 4), KARGS);
  };
  gload(0);
  sload(sl, 0);
  lstore(0);
  __syncthreads();
  for (int jt = 0; jt < nj; ++jt) {
    const int buf = jt & 1;
    const idx_t j0 = (idx_t)jt * BJ;
    if (jt + 1 < nj) gload(j0 + BJ);
    sload(sl_next, jt + 1 < nj ? j0 + BJ : j0);          // a step ahead, like the key / value tiles

    // ---- S^T = K . Q^T for 64 keys x this wavefront's 32 queries
    f32x16 sacc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[t][e] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const frag_t a = __builtin_bit_cast(frag_t, *(const u16x8*)&Ks[buf][t * 32 + l31][ks * 16 + h * 8]);
        sacc[t] = MFMA(a, rq[ks], sacc[t], 0, 0, 0);
      }
    }
    // ---- the block's One-to-One operators on the scores; accumulator element e of tile t is key
    //      j0 + 32 t + 8 (e / 4) + 4 h + e % 4 of query qi
    float mx = -__builtin_inff();
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float s4[4] = {sacc[t][4 * q], sacc[t][4 * q + 1], sacc[t][4 * q + 2], sacc[t][4 * q + 3]};
        const idx_t jq = j0 + t * 32 + q * 8 + h * 4;
        score4(z, qic, KEY4(jq), sl[t][q], s4, KARGS);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (SK % BJ != 0 && jq + u >= SK) s4[u] = -__builtin_inff();
          sacc[t][4 * q + u] = s4[u];
          mx = fmaxf(mx, s4[u]);
        }
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));            // the other half-wave holds the same query's other keys
    // The reference value the exponentials are taken against only has to stay within a safe distance of
    // the running maximum, not equal it: it moves when some row's maximum has grown by more than
    // 2^8 (probabilities then reach at most 256, harmless in fp32 sums and in the 16-bit operand), and
    // only then are the partial sums and the output accumulators rescaled.  After a row's first tiles
    // that is rare, so the common step has no rescaling work.
    const float cand = fmaxf(m_run, mx);
    const bool move = (cand - m_run) * LOG2E > 8.0f;      // also true for the first finite maximum (m_run = -inf)
    if (__builtin_amdgcn_ballot_w64(move) != 0) {
      const float m_next = move ? cand : m_run;
      const float alpha = m_next == m_run ? 1.0f : dn_exp2((m_run - m_next) * LOG2E);   // exp2(-inf) = 0 on the first move
      m_run = m_next;
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < TD; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
    }
    const float m2 = (m_run == -__builtin_inff() ? 0.0f : m_run) * LOG2E;   // a row with nothing but -inf so far
    float psum = 0.0f;
    frag_t pf[4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        pelem_t pv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float p = dn_exp2(__builtin_fmaf(sacc[t][half * 8 + u], LOG2E, -m2));
          psum += p;                                     // the row sum keeps fp32; the MFMA operand is rounded (RNE)
          pv[u] = (pelem_t)p;
        }
        pf[t * 2 + half] = (frag_t){pv[0], pv[1], pv[2], pv[3], pv[4], pv[5], pv[6], pv[7]};
      }
    l_run += psum;
    // ---- O^T += V^T . P^T
#pragma unroll
    for (int t = 0; t < TD; ++t) {
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const frag_t a = __builtin_bit_cast(frag_t, *(const u16x8*)&Vt[buf][t * 32 + l31][st * 16 + h * 8]);
        oacc[t] = MFMA(a, pf[st], oacc[t], 0, 0, 0);
      }
    }
    if (jt + 1 < nj) lstore(buf ^ 1);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) sl[t][q] = sl_next[t][q];
    __syncthreads();
  }

  // ---- normalise, then the second MatMul's epilogue through LDS (lanes along the output columns)
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  float* Cs = (float*)smem;                              // every wavefront is past its last tile read
#pragma unroll
  for (int t = 0; t < TD; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) Cs[(wave * 32 + l31) * CLD + t * 32 + 8 * (e >> 2) + 4 * h + (e & 3)] = oacc[t][e] * inv;
  __syncthreads();
#if EPI_VEC > 1
  for (int idx = tid; idx < BQ * (DV / EPI_VEC); idx += 256) {
    const int rl = idx / (DV / EPI_VEC), c_l = (idx % (DV / EPI_VEC)) * EPI_VEC;
    float v[EPI_VEC];
#pragma unroll
    for (int u = 0; u < EPI_VEC; u += 4) {
      const f32x4 t4 = *(const f32x4*)&Cs[rl * CLD + c_l + u];
      v[u] = t4[0]; v[u + 1] = t4[1]; v[u + 2] = t4[2]; v[u + 3] = t4[3];
    }
    if (q0 + rl < SQ) epilogue_vec(z, q0 + rl, c_l, v, KARGS);
  }
#else
  for (int idx = tid; idx < BQ * DV; idx += 256) {
    const int rl = idx / DV, c_l = idx % DV;
    if (q0 + rl < SQ) {
      float cv[NCOLV > 0 ? NCOLV : 1];
      col_loads(c_l, cv, KARGS);
      epilogue(z, q0 + rl, c_l, Cs[rl * CLD + c_l], cv, KARGS);
    }
  }
#endif
}
)KRN";

}  // namespace

Lowered lower_attention(const Graph& g, const Block& b, const LowerOpts& o) {
  // ---- the three anchors
  int sm = -1;
  std::vector<int> mms;
  for (int oi : b.ops) {
    if (g.ops[oi].info->cls == OC_SOFTMAX) { DNNF_CHECK(sm < 0, DNNF_UNSUPPORTED_OP, "two Softmax operators in one block"); sm = oi; }
    if (g.ops[oi].info->cls == OC_MATMUL) mms.push_back(oi);
  }
  DNNF_CHECK(sm >= 0 && mms.size() == 2, DNNF_UNSUPPORTED_OP, "not a MatMul - Softmax - MatMul block");
  const Op& SM = g.ops[sm];
  const int X = SM.in[0], P = SM.out[0];
  const Tensor& TX = g.tensors[X];
  int64_t axis = SM.i("axis", -1);
  if (axis < 0) axis += (int64_t)TX.dims.size();
  DNNF_CHECK(axis == (int64_t)TX.dims.size() - 1, DNNF_UNSUPPORTED_OP, "Softmax over an axis other than the last");
  // operators the Softmax input depends on (inside the block) form the score part
  std::set<int> in_block(b.ops.begin(), b.ops.end()), score_ops;
  {
    std::vector<int> stack = {X};
    while (!stack.empty()) {
      int t = stack.back();
      stack.pop_back();
      int p = g.tensors[t].producer;
      if (p < 0 || !in_block.count(p) || score_ops.count(p)) continue;
      score_ops.insert(p);
      for (int i : g.ops[p].in) stack.push_back(i);
    }
  }
  int mm1 = -1, mm2 = -1;
  for (int m : mms) (score_ops.count(m) ? mm1 : mm2) = m;
  DNNF_CHECK(mm1 >= 0 && mm2 >= 0 && mm1 != mm2, DNNF_UNSUPPORTED_OP, "the two MatMul operators must sit on either side of the Softmax");
  DNNF_CHECK(g.ops[mm2].in[0] == P && g.tensors[P].consumers.size() == 1 && g.tensors[P].kind == DNNF_INTERMEDIATE,
             DNNF_UNSUPPORTED_OP, "the probabilities must feed the second MatMul's first operand and nothing else");
  Block bs, bo;
  for (int oi : b.ops) {
    if (oi == sm) continue;
    (score_ops.count(oi) ? bs : bo).ops.push_back(oi);
  }
  bs.fused_type = bo.fused_type = DNNF_MANY_TO_MANY;

  LowerCtx cs(g, bs, o), co(g, bo, o);
  cs.anchor_op = mm1;
  cs.anchor_out = g.ops[mm1].out[0];
  co.anchor_op = mm2;
  co.anchor_out = g.ops[mm2].out[0];
  for (int oi : bs.ops)
    DNNF_CHECK(oi == mm1 || (g.ops[oi].info->cls != OC_REDUCE && g.ops[oi].info->cls != OC_SOFTMAX && g.ops[oi].info->cls != OC_NORMALIZE &&
                             g.ops[oi].info->cls != OC_GAP && g.ops[oi].info->cls != OC_CONV),
               DNNF_UNSUPPORTED_OP, "a second Many-to-Many operator among the score operators");
  for (int oi : bo.ops)
    DNNF_CHECK(oi == mm2 || (g.ops[oi].info->cls != OC_REDUCE && g.ops[oi].info->cls != OC_SOFTMAX && g.ops[oi].info->cls != OC_NORMALIZE &&
                             g.ops[oi].info->cls != OC_GAP && g.ops[oi].info->cls != OC_CONV && g.ops[oi].info->cls != OC_MATMUL),
               DNNF_UNSUPPORTED_OP, "a further Many-to-Many operator behind the second MatMul");
  MatmulFrame fs = analyse_matmul(cs), fo = analyse_matmul(co);

  const int dtype = fs.dtype;
  DNNF_CHECK(dtype_bytes(dtype) == 2 && fo.dtype == dtype, DNNF_UNSUPPORTED_OP, "the attention template needs 16-bit operands");
  const int64_t SQ = fs.GM, SK = fs.GN, DH = fs.K, DV = fo.GN, GZ = fs.GZ;
  DNNF_CHECK(fo.GM == SQ && fo.K == SK && fo.GZ == GZ, DNNF_UNSUPPORTED_OP, "the two MatMul operators do not share rows / batch");
  DNNF_CHECK(DH % 16 == 0 && DH <= 128 && DV % 32 == 0 && DV <= 128, DNNF_UNSUPPORTED_OP, "head dimension outside the template's range");
  DNNF_CHECK(SK % 8 == 0, DNNF_UNSUPPORTED_OP, "key count must be a multiple of 8");
  // the same (batch, query) numbering on both sides
  auto extents = [](const LowerCtx& c, const std::vector<int>& v) {
    std::vector<int64_t> e;
    for (int a : v) e.push_back(c.atom_extent[a]);
    return e;
  };
  DNNF_CHECK(extents(cs, fs.batch) == extents(co, fo.batch) && extents(cs, fs.rows) == extents(co, fo.rows), DNNF_UNSUPPORTED_OP,
             "batch / query axes of the two MatMul operators are ordered differently");
  // Softmax runs over the score columns, rows and batch are untouched by the score operators
  DNNF_CHECK(cs.stores.size() == 1 && cs.stores[0].tensor == X && cs.stores[0].preds.empty(), DNNF_UNSUPPORTED_OP,
             "a score intermediate is read outside the block");
  {
    const TIdx& xi = cs.tidx.at(X);
    std::vector<int> last;
    cs.resolve(xi.back().atoms, last);
    DNNF_CHECK(last == fs.cols && xi.back().offset == 0 && xi.back().indirect < 0, DNNF_UNSUPPORTED_OP, "Softmax axis is not the key axis");
    std::vector<int> lead;
    for (size_t d = 0; d + 1 < xi.size(); d++) { DNNF_CHECK(xi[d].offset == 0 && xi[d].indirect < 0, DNNF_UNSUPPORTED_OP, "sliced scores"); cs.resolve(xi[d].atoms, lead); }
    std::vector<int> want = fs.batch;
    want.insert(want.end(), fs.rows.begin(), fs.rows.end());
    DNNF_CHECK(lead == want, DNNF_UNSUPPORTED_OP, "score operators permute the batch / query axes");
  }
  DNNF_CHECK(fs.amode == 0, DNNF_UNSUPPORTED_OP, "queries must be contiguous along the head dimension");
  DNNF_CHECK(fs.bmode == 0 || fs.bmode == 1, DNNF_UNSUPPORTED_OP, "keys need a vectorisable layout");
  DNNF_CHECK(fo.bmode == 0 || fo.bmode == 1, DNNF_UNSUPPORTED_OP, "values need a vectorisable layout");
  const int inner = fs.cols.back();
  DNNF_CHECK(cs.atom_extent[inner] % 4 == 0, DNNF_UNSUPPORTED_OP, "key axis split too finely");

  // ---- parameters: Q, K, V, what the score operators read, what the epilogue reads, outputs
  std::vector<int> params = {fs.ta, fs.tb, fo.tb};
  std::map<int, int> pslot;
  std::set<int> written;
  auto collect = [&](const LowerCtx& c, std::set<int>& need) {
    std::vector<int> stack;
    for (auto& s : c.stores) stack.push_back(s.value);
    while (!stack.empty()) {
      int n = stack.back();
      stack.pop_back();
      if (need.count(n)) continue;
      need.insert(n);
      for (int a : c.nodes[n].args) stack.push_back(a);
      if (c.nodes[n].kind == ENode::LOAD) {
        DNNF_CHECK(c.nodes[n].addr.indirect.empty(), DNNF_UNSUPPORTED_OP, "gathered operand in an attention block");
        if (!pslot.count(c.nodes[n].tensor)) { pslot[c.nodes[n].tensor] = (int)params.size(); params.push_back(c.nodes[n].tensor); }
      }
    }
  };
  std::set<int> need_s, need_o;
  collect(cs, need_s);
  collect(co, need_o);
  size_t n_in = params.size();
  for (auto& s : co.stores) {
    DNNF_CHECK(!pslot.count(s.tensor) && s.tensor != fs.ta && s.tensor != fs.tb && s.tensor != fo.tb, DNNF_UNSUPPORTED_OP,
               "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }
  bool wide = false;
  for (int t : params) wide = wide || g.tensors[t].n() >= (int64_t)1 << 31;
  wide = wide || GZ * SQ * SK >= (int64_t)1 << 31;

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "typedef " << cs.ctype(dtype) << " elem_t;\n";
  k << "#define SQ " << SQ << "\n#define SK " << SK << "\n#define DH " << DH << "\n#define DV " << DV << "\n";
  k << "#define K_MODE " << fs.bmode << "\n#define V_MODE " << fo.bmode << "\n#define PQ p0\n#define PK p1\n#define PV p2\n";
  if (dtype == DNNF_F16) k << "typedef f16x8 frag_t;\ntypedef _Float16 pelem_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16\n";
  else k << "typedef bf16x8 frag_t;\ntypedef __bf16 pelem_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16\n";
  k << gemm_offset_fn(cs, "offQ_row", fs.rows, fs.aa) << gemm_offset_fn(cs, "offQ_k", fs.katoms, fs.aa) << gemm_offset_fn(cs, "offQ_batch", fs.batch, fs.aa);
  k << gemm_offset_fn(cs, "offK_col", fs.cols, fs.ab) << gemm_offset_fn(cs, "offK_k", fs.katoms, fs.ab) << gemm_offset_fn(cs, "offK_batch", fs.batch, fs.ab);
  k << gemm_offset_fn(co, "offV_col", fo.cols, fo.ab) << gemm_offset_fn(co, "offV_k", fo.katoms, fo.ab) << gemm_offset_fn(co, "offV_batch", fo.batch, fo.ab);
  std::string kparams = cs.param_list(params, written), kargs;
  for (size_t i = 0; i < params.size(); i++) kargs += (i ? ", p" : "p") + std::to_string(i);

  // ---- score function: the block's operators between the first MatMul and the Softmax, four keys at a time
  {
    // Operands that run along the keys (masks) are fetched by a function of their own, four keys per
    // vector, so that the kernel can issue the loads of the next key tile a whole step ahead.
    std::map<int, std::string> ov;
    std::vector<int> vloads;
    for (int n : need_s) {
      const ENode& e = cs.nodes[n];
      if (e.kind != ENode::LOAD || e.is_int) continue;
      Affine a = cs.resolved(e.addr);
      bool contig = stride_of(a, inner) == 1 && a.offset % 4 == 0;
      for (auto& kv : a.stride) if (kv.first != inner && kv.second % 4) contig = false;
      if (!contig) continue;
      vloads.push_back(n);
      ov[n] = "cvt_in(L.lv" + std::to_string(n) + "[u])";
    }
    for (int n : vloads)
      k << "typedef " << cs.ctype(g.tensors[cs.nodes[n].tensor].dtype) << " lv" << n << "_t __attribute__((ext_vector_type(4)));\n";
    k << "struct sload_t {\n";
    for (int n : vloads) k << "  lv" << n << "_t lv" << n << ";\n";
    if (vloads.empty()) k << "  int none;\n";
    k << "};\n";
    k << "DEV sload_t score_load(idx_t z, idx_t r, idx_t cc, " << kparams << ") {\n";
    decl_digits(k, cs, fs.batch, "z", "  ", "qz");
    decl_digits(k, cs, fs.rows, "r", "  ", "qr");
    decl_digits(k, cs, fs.cols, "cc", "  ", "qc");
    k << "  sload_t L;\n";
    for (int n : vloads) {
      const ENode& e = cs.nodes[n];
      k << "  L.lv" << n << " =*(const lv" << n << "_t*)(p" << pslot.at(e.tensor) << " + (" << cs.addr_expr(e.addr) << "));\n";
    }
    if (vloads.empty()) k << "  L.none = 0;\n";
    k << "  return L;\n}\n";
    k << "DEV void score4(idx_t z, idx_t r, idx_t cc, const sload_t L, float* s, " << kparams << ") {\n";
    decl_digits(k, cs, fs.batch, "z", "  ", "qz");
    decl_digits(k, cs, fs.rows, "r", "  ", "qr");
    decl_digits(k, cs, fs.cols, "cc", "  ", "qc");
    k << "  const idx_t inner0 = a" << inner << ";\n";
    k << "#pragma unroll\n  for (int u = 0; u < 4; ++u) {\n";
    k << "    const idx_t a" << inner << " = inner0 + u;\n    const float anchor_v = s[u];\n";
    std::set<int> done;
    cs.emit_values(k, {cs.stores[0].value}, done, pslot, "    ", &ov);
    k << "    s[u] = " << cs.vname(cs.stores[0].value) << ";\n  }\n}\n";
  }
  // ---- epilogue of the second MatMul (rows = queries, columns = value channels)
  k << gemm_epilogue_source(co, fo.batch, fo.rows, fo.cols, pslot, kparams, DV, -1);
  k << "#define KPARAMS " << kparams << "\n#define KARGS " << kargs << "\n";
  k << kAttnBody;

  Lowered Lw;
  Lw.family = FAM_ATTENTION;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch Kn;
  Kn.params = params;
  Kn.grid[0] = (unsigned)(GZ * ((SQ + 127) / 128));
  Kn.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_attn", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  Lw.variant = "stream_softmax_128x64_d" + std::to_string(DH) + "_k" + std::to_string(fs.bmode) + "v" + std::to_string(fo.bmode);
  return Lw;
}

}  // namespace dnnf
