// fs_device.h - device-side building blocks of stitched kernels for gfx950 (CDNA4, wave64).
//
// A stitched kernel is a generated straight-line body that calls the pieces below.  The
// body is the paper's thread composition (Section 1, Figure 2(a)): every elementwise node of
// the fused group is evaluated in registers on the lane's slice of a row.  Nodes that need
// another parallel loop - reductions and whatever consumes them - are joined inside the same
// kernel through on-chip memory, the paper's block composition (Section 1, Figure 2(b);
// Section 5.2, Algorithm 2).  On this hardware a 64-lane wavefront exchanges values through
// DPP / lane-permute instructions without touching LDS at all, so LDS is only needed when a
// row spans several wavefronts, for column partials and for transposing stores.
//
// Work decomposition (a Row schedule with split_dim = 0 in the terms of Section 4.1): a
// workgroup of WG lanes is split into G = WG / L row-groups of L lanes.  Per loop trip a
// row-group owns one row; lane `lir` of the row-group owns the 16-byte vectors
// j*L + lir (j = 0..NVL-1) of that row, i.e. E = NVL*V elements that stay in VGPRs for the
// whole body.  Consecutive lanes touch consecutive 16-byte vectors: every wave-wide memory
// instruction is fully coalesced.
//
// This header is compiled two ways: ahead of time with hipcc (to check it and for the
// probe kernels) and at run time as the prefix of every generated kernel.
#ifndef FS_DEVICE_H_
#define FS_DEVICE_H_

#define FS_DEV __device__ __forceinline__

// dtype tags (values match the host enum fs_dtype)
#define FS_DT_F32 0
#define FS_DT_BF16 1
#define FS_DT_U8 2
// reduction kinds (values match fs_reduce_kind)
#define FS_K_SUM 0
#define FS_K_MAX 1
#define FS_K_MIN 2
#define FS_K_MEAN 3

typedef unsigned int fs_u32;
typedef unsigned short fs_u16;
typedef unsigned char fs_u8;

template <int DT> struct fs_elem;
template <> struct fs_elem<FS_DT_F32> { typedef float type; };
template <> struct fs_elem<FS_DT_BF16> { typedef fs_u16 type; };
template <> struct fs_elem<FS_DT_U8> { typedef fs_u8 type; };

template <typename T, int N> struct fs_vec { typedef T type __attribute__((ext_vector_type(N))); };
template <typename T> struct fs_vec<T, 1> { typedef T type; };

// ------------------------------------------------------------------------------------------
// scalar conversions
// ------------------------------------------------------------------------------------------
FS_DEV constexpr float fs_lit(fs_u32 bits) { return __builtin_bit_cast(float, bits); }  // exact literal
FS_DEV float fs_bf16_bits_to_f32(fs_u16 h) { return __builtin_bit_cast(float, (fs_u32)h << 16); }
// round-to-nearest-even fp32 -> bf16 (v_cvt_pk_bf16_f32 on gfx950)
FS_DEV fs_u16 fs_f32_to_bf16_bits(float f) { return __builtin_bit_cast(fs_u16, (__bf16)f); }

template <int DT> FS_DEV float fs_to_f32(typename fs_elem<DT>::type x);
template <> FS_DEV float fs_to_f32<FS_DT_F32>(float x) { return x; }
template <> FS_DEV float fs_to_f32<FS_DT_BF16>(fs_u16 x) { return fs_bf16_bits_to_f32(x); }
template <> FS_DEV float fs_to_f32<FS_DT_U8>(fs_u8 x) { return x ? 1.0f : 0.0f; }

template <int DT> FS_DEV typename fs_elem<DT>::type fs_from_f32(float x);
template <> FS_DEV float fs_from_f32<FS_DT_F32>(float x) { return x; }
template <> FS_DEV fs_u16 fs_from_f32<FS_DT_BF16>(float x) { return fs_f32_to_bf16_bits(x); }
template <> FS_DEV fs_u8 fs_from_f32<FS_DT_U8>(float x) { return x != 0.0f ? (fs_u8)1 : (fs_u8)0; }

// A node's value is rounded once to its declared dtype even when it never leaves registers.
template <int DT> FS_DEV float fs_round(float x) { return x; }
template <> FS_DEV float fs_round<FS_DT_BF16>(float x) { return fs_bf16_bits_to_f32(fs_f32_to_bf16_bits(x)); }

// ------------------------------------------------------------------------------------------
// elementwise math.  + - * / sqrt max min are the IEEE operations (the translation unit is
// compiled without contraction), so values that feed a predicate are reproducible bit for bit.
// exp/log/tanh/sigmoid/gelu/rsqrt/rcp are built on the hardware's 1-ulp transcendental
// instructions (v_exp_f32, v_log_f32, v_rcp_f32, v_rsq_f32).
// ------------------------------------------------------------------------------------------
#define FS_LOG2E 1.4426950408889634f
#define FS_LN2 0.6931471805599453f

// exp(x) = 2^(x*log2e).  The product is carried in two floats (t + r) so its rounding error
// does not grow with |x|: 2^(t+r) = 2^t * (1 + r ln2 + ...).
FS_DEV float fs_exp(float x) {
  const float t = x * FS_LOG2E;
  float r = __builtin_fmaf(x, FS_LOG2E, -t);
  r = __builtin_fmaf(x, 1.925963033500494e-8f /* log2(e) - float(log2(e)) */, r);
  const float p = __builtin_amdgcn_exp2f(t);
  return __builtin_fmaf(p, r * FS_LN2, p);
}
FS_DEV float fs_log(float x) { return __builtin_amdgcn_logf(x) * FS_LN2; }
FS_DEV float fs_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
FS_DEV float fs_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }
FS_DEV float fs_sqrt(float x) { return __builtin_sqrtf(x); }
FS_DEV float fs_div(float a, float b) { return a / b; }
FS_DEV float fs_max(float a, float b) { return __builtin_fmaxf(a, b); }
FS_DEV float fs_min(float a, float b) { return __builtin_fminf(a, b); }

// sigmoid(x) = 1 / (1 + 2^(-x log2e)); saturates cleanly to 0 and 1.
FS_DEV float fs_sigmoid(float x) {
  const float e = __builtin_amdgcn_exp2f(x * -FS_LOG2E);
  return __builtin_amdgcn_rcpf(1.0f + e);
}

// tanh: for |x| >= 1/4, 1 - 2/(e^{2|x|}+1) (no cancellation there); below, the odd Maclaurin
// polynomial through x^9 (truncation < 1e-8 relative at 1/4).  Both sides are evaluated and
// selected, so a wave never diverges.
FS_DEV float fs_tanh(float x) {
  const float ax = __builtin_fabsf(x);
  const float e = __builtin_amdgcn_exp2f(ax * (2.0f * FS_LOG2E));
  const float big = __builtin_fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
  const float x2 = x * x;
  float p = __builtin_fmaf(x2, 0.021869488536155203f, -0.053968253968253971f);
  p = __builtin_fmaf(x2, p, 0.13333333333333333f);
  p = __builtin_fmaf(x2, p, -0.33333333333333331f);
  const float small = __builtin_fmaf(ax * x2, p, ax);
  return __builtin_copysignf(ax < 0.25f ? small : big, x);
}

// tanh-GeLU: 0.5 z (1 + tanh(u)) with u = sqrt(2/pi) (z + 0.044715 z^3).  Since
// (1 + tanh u)/2 = sigmoid(2u), it is evaluated as z / (1 + 2^(-2u log2e)): no cancellation in
// the negative tail, one exp and one rcp per element.  The constants of u and of the base-2
// exponent are folded into one odd polynomial: -2u log2e = z (c2 + c1 z^2).
FS_DEV float fs_gelu_tanh(float z) {
  constexpr float c2 = -2.0f * 0.7978845608028654f * FS_LOG2E;
  constexpr float c1 = 0.044715f * c2;
  const float t = __builtin_fmaf(c1, z * z, c2);
  const float e = __builtin_amdgcn_exp2f(z * t);
  return z * __builtin_amdgcn_rcpf(1.0f + e);
}

// ------------------------------------------------------------------------------------------
// vector memory access: V elements of dtype DT per access (16 bytes for the widest dtype of
// the group).  Invalid rows / columns load zeros and store nothing.
// ------------------------------------------------------------------------------------------
template <int DT, int V, bool NT = false> FS_DEV void fs_load_vec(float* dst, const void* base, long elem_index) {
  typedef typename fs_elem<DT>::type T;
  typedef typename fs_vec<T, V>::type VT;
  const VT* p = reinterpret_cast<const VT*>(static_cast<const T*>(base) + elem_index);
  const VT raw = NT ? __builtin_nontemporal_load(p) : *p;
  if constexpr (V == 1) {
    dst[0] = fs_to_f32<DT>(raw);
  } else {
#pragma unroll
    for (int k = 0; k < V; ++k) dst[k] = fs_to_f32<DT>(raw[k]);
  }
}

template <int DT, int V, bool NT = false> FS_DEV void fs_store_vec(const float* src, void* base, long elem_index) {
  typedef typename fs_elem<DT>::type T;
  typedef typename fs_vec<T, V>::type VT;
  VT raw;
  if constexpr (V == 1) {
    raw = fs_from_f32<DT>(src[0]);
  } else {
#pragma unroll
    for (int k = 0; k < V; ++k) raw[k] = fs_from_f32<DT>(src[k]);
  }
  VT* p = reinterpret_cast<VT*>(static_cast<T*>(base) + elem_index);
  if constexpr (NT) __builtin_nontemporal_store(raw, p);
  else *p = raw;
}

// Load the lane's slice of one row tile: vectors vbase + j*L + lir, j < NVL (vbase = 0 unless a
// row is cut into several column tiles).  `row_elem0` is the element index of the first column
// of a VALID row (callers clamp the row index instead of predicating the load).  NV = vectors
// per row; RAGGED says some of those vector indices can fall beyond NV: they are clamped too.
// Nothing here branches, so all loads of a body are issued back to back and waited for once;
// lanes outside the tensor hold duplicates that are never stored and never reduced.
// (the _vec forms handle vector j of the slice alone: a body that is emitted vector by vector
// keeps fewer registers live)
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, bool NT = false>
FS_DEV void fs_load_row_vec(float (&dst)[NVL * V], const void* base, long row_elem0, int lir, int vbase, int j) {
  int vi = vbase + j * L + lir;
  if (RAGGED) vi = vi < NV ? vi : NV - 1;
  fs_load_vec<DT, V, NT>(&dst[j * V], base, row_elem0 + (long)vi * V);
}
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, bool NT = false>
FS_DEV void fs_load_row(float (&dst)[NVL * V], const void* base, long row_elem0, int lir, int vbase) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) fs_load_row_vec<DT, V, NVL, L, NV, RAGGED, NT>(dst, base, row_elem0, lir, vbase, j);
}

// The lane's slice of a row that is the concatenation of two tensors in memory.  AXIS 1 (columns): a is [R,SPLIT],
// b is [R,CB], the row is a's row followed by b's (SPLIT and CB are multiples of V: no vector straddles the seam).
// AXIS 0 (rows): rows below SPLIT come from a, the others from b, both NV*V columns wide.  The source is chosen
// by selecting the address, not by branching: every lane issues exactly one load per vector.
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, int AXIS, long SPLIT, long CB>
FS_DEV void fs_load_row_concat(float (&dst)[NVL * V], const void* a, const void* b, long row, int lir, int vbase) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) {
    int vi = vbase + j * L + lir;
    if (RAGGED) vi = vi < NV ? vi : NV - 1;
    const long col = (long)vi * V;
    const bool first = AXIS == 1 ? col < SPLIT : row < SPLIT;
    const long idx = AXIS == 1 ? (first ? row * SPLIT + col : row * CB + (col - SPLIT)) : (first ? row : row - SPLIT) * ((long)NV * V) + col;
    fs_load_vec<DT, V>(&dst[j * V], first ? a : b, idx);
  }
}

template <int DT, int V, int NVL, int L, int NV, bool RAGGED, bool NT = false>
FS_DEV void fs_store_row_vec(const float (&src)[NVL * V], void* base, long row_elem0, int lir, int vbase, bool rok, int j) {
  const int vi = vbase + j * L + lir;
  const bool ok = rok && (!RAGGED || vi < NV);
  if (ok) fs_store_vec<DT, V, NT>(&src[j * V], base, row_elem0 + (long)vi * V);
}
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, bool NT = false>
FS_DEV void fs_store_row(const float (&src)[NVL * V], void* base, long row_elem0, int lir, int vbase, bool rok) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) fs_store_row_vec<DT, V, NVL, L, NV, RAGGED, NT>(src, base, row_elem0, lir, vbase, rok, j);
}

// One chunk of a row kept in LDS in the tensor's own dtype (a kernel that walks a row once per stage reads the
// chunk from memory in the first stage only).  The lane's vector j sits at chunk-local vector j*L + lir: consecutive
// lanes touch consecutive 16-byte pieces.  What is written is what fs_load_row delivered (fp32 values that came from
// the dtype convert back to it exactly), clamped duplicates included, so a later read sees the very same registers.
template <int DT, int V, int NVL, int L> FS_DEV void fs_stage_row_chunk(void* lds_chunk, const float (&src)[NVL * V], int lir) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) fs_store_vec<DT, V>(&src[j * V], lds_chunk, (long)(j * L + lir) * V);
}
// fs_load_row and fs_stage_row_chunk in one: the vectors go to LDS as they came from memory (when `stage`), so nothing is
// spent on converting fp32 registers back to the dtype, and what a later stage reads back is the same bytes.
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, bool NT = false>
FS_DEV void fs_load_row_staging(float (&dst)[NVL * V], const void* base, long row_elem0, int lir, int vbase, void* lds_chunk, bool stage) {
  typedef typename fs_elem<DT>::type T;
  typedef typename fs_vec<T, V>::type VT;
#pragma unroll
  for (int j = 0; j < NVL; ++j) {
    int vi = vbase + j * L + lir;
    if (RAGGED) vi = vi < NV ? vi : NV - 1;
    const VT* p = reinterpret_cast<const VT*>(static_cast<const T*>(base) + row_elem0 + (long)vi * V);
    const VT raw = NT ? __builtin_nontemporal_load(p) : *p;
    if (stage) *reinterpret_cast<VT*>(static_cast<T*>(lds_chunk) + (long)(j * L + lir) * V) = raw;
    if constexpr (V == 1) {
      dst[j] = fs_to_f32<DT>(raw);
    } else {
#pragma unroll
      for (int k = 0; k < V; ++k) dst[j * V + k] = fs_to_f32<DT>(raw[k]);
    }
  }
}
template <int DT, int V, int NVL, int L> FS_DEV void fs_load_row_chunk_lds(float (&dst)[NVL * V], const void* lds_chunk, int lir) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) fs_load_vec<DT, V>(&dst[j * V], lds_chunk, (long)(j * L + lir) * V);
}

// Transposing store of the lane's slice of row `row` of a [R,C] value into a [C,R] tensor.
template <int DT, int V, int NVL, int L, int NV, bool RAGGED>
FS_DEV void fs_store_row_transposed(const float (&src)[NVL * V], void* base, long R, long row, int lir, int vbase, bool rok) {
  typedef typename fs_elem<DT>::type T;
#pragma unroll
  for (int j = 0; j < NVL; ++j) {
    const int vi = vbase + j * L + lir;
    const bool ok = rok && (!RAGGED || vi < NV);
    if (ok) {
#pragma unroll
      for (int k = 0; k < V; ++k) static_cast<T*>(base)[(long)(vi * V + k) * R + row] = fs_from_f32<DT>(src[j * V + k]);
    }
  }
}

// Per-column vectors ([1,C] operands) shared by every row of the workgroup are staged once in
// LDS as fp32: one cooperative pass of the whole workgroup instead of every wavefront pulling
// its own copy through the vector cache (which is the narrower path: 64 B/clk against 128).
// The staged copy is laid out in the order lanes read it: the 4-float chunk q of vector
// vi = j*L + lir sits at chunk index (j*(V/4) + q)*L + lir, so a 128-bit LDS read by
// consecutive lanes touches consecutive 16-byte chunks (no bank conflicts).  The staging pass
// walks the LDS positions in order (thread t writes position t, t + WG, ...), so its 128-bit
// writes are conflict-free too; what it reads from memory is then 16-byte pieces V*4 bytes
// apart, a few KB from L2 once per workgroup.  SLOT = NVL*L*V floats per vector.
template <int DT, int V, int L, int C, int WG> FS_DEV void fs_stage_rowvec(float* lds, const void* src) {
  if constexpr (V % 4 == 0) {
    constexpr int Q = V / 4, NVS = C / V;  // 16-byte pieces per vector access, vectors per row
    constexpr int P = ((NVS + L - 1) / L) * Q * L;  // LDS positions (16-byte pieces) of the slot, tail included
    for (int p = (int)threadIdx.x; p < P; p += WG) {
      const int l = p % L, jq = p / L, j = jq / Q, q = jq % Q, vi = j * L + l;
      if (vi >= NVS) continue;
      float tmp[4];
      fs_load_vec<DT, 4>(tmp, src, (vi * Q + q) * 4);
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 t4;
#pragma unroll
      for (int k = 0; k < 4; ++k) t4[k] = tmp[k];
      *reinterpret_cast<f4*>(lds + p * 4) = t4;  // one 128-bit LDS store, consecutive threads to consecutive pieces
    }
  } else {
    for (int i = (int)threadIdx.x; i < C; i += WG) {
      float tmp[1];
      fs_load_vec<DT, 1>(tmp, src, i);
      lds[i] = tmp[0];
    }
  }
}
// The same for the sum (or difference) of two per-column vectors: +-a +- b is formed once, here,
// instead of once per element of every row.
template <int DTA, int DTB, bool NEGA, bool NEGB, int V, int L, int C, int WG> FS_DEV void fs_stage_rowvec_sum(float* lds, const void* a, const void* b) {
  if constexpr (V % 4 == 0) {
    constexpr int Q = V / 4, NVS = C / V;
    constexpr int P = ((NVS + L - 1) / L) * Q * L;
    for (int p = (int)threadIdx.x; p < P; p += WG) {
      const int l = p % L, jq = p / L, j = jq / Q, q = jq % Q, vi = j * L + l;
      if (vi >= NVS) continue;
      float ta[4], tb[4];
      fs_load_vec<DTA, 4>(ta, a, (vi * Q + q) * 4);
      fs_load_vec<DTB, 4>(tb, b, (vi * Q + q) * 4);
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 t4;
#pragma unroll
      for (int k = 0; k < 4; ++k) t4[k] = (NEGA ? -ta[k] : ta[k]) + (NEGB ? -tb[k] : tb[k]);
      *reinterpret_cast<f4*>(lds + p * 4) = t4;
    }
  } else {
    for (int i = (int)threadIdx.x; i < C; i += WG) {
      float ta[1], tb[1];
      fs_load_vec<DTA, 1>(ta, a, i);
      fs_load_vec<DTB, 1>(tb, b, i);
      lds[i] = (NEGA ? -ta[0] : ta[0]) + (NEGB ? -tb[0] : tb[0]);
    }
  }
}
// The lane's slice of a staged vector (same element ownership as fs_load_row).
template <int V, int NVL, int L, int NV, bool RAGGED>
FS_DEV void fs_read_staged_vec(float (&dst)[NVL * V], const float* lds, int lir, int j) {
  if constexpr (V % 4 == 0) {
    constexpr int Q = V / 4;
    typedef float f4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const f4 x = *reinterpret_cast<const f4*>(lds + ((j * Q + q) * L + lir) * 4);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float xk = x[k];
        dst[j * V + q * 4 + k] = xk;
      }
    }
  } else {
    int vi = j * L + lir;
    if (RAGGED) vi = vi < NV ? vi : NV - 1;
#pragma unroll
    for (int k = 0; k < V; ++k) dst[j * V + k] = lds[vi * V + k];
  }
}
template <int V, int NVL, int L, int NV, bool RAGGED>
FS_DEV void fs_read_staged(float (&dst)[NVL * V], const float* lds, int lir) {
#pragma unroll
  for (int j = 0; j < NVL; ++j) fs_read_staged_vec<V, NVL, L, NV, RAGGED>(dst, lds, lir, j);
}

template <int DT> FS_DEV void fs_store1_fwd(void* base, long i, float x) {
  static_cast<typename fs_elem<DT>::type*>(base)[i] = fs_from_f32<DT>(x);
}

// Transposing store of a G x TC tile (one row per row-group, in registers) through a padded LDS
// tile: rows tile_row0 .. tile_row0+G-1 and columns col0 .. col0+TC-1 of the [R,CTOT] value become
// G consecutive elements of each of TC rows of the [CTOT,R] output, so global stores are runs of G
// elements instead of single elements R apart.  LDS holds TC x (G+1) floats (the +1 keeps the
// column-wise writes of the row-groups of a wavefront on distinct banks).  vbase = col0 / V is the
// tile's first vector in the row.  Every lane of the workgroup must call it.
template <int DT, int V, int NVL, int L, int NV, bool RAGGED, int WG, int TC, int CTOT, bool NT = false>
FS_DEV void fs_store_tile_transposed(const float (&src)[NVL * V], float* lds, void* base, long R, long tile_row0, int lir, int rg, int vbase) {
  constexpr int G = WG / L, P = G + 1;
  __syncthreads();  // the tile may still be read by its previous use
#pragma unroll
  for (int j = 0; j < NVL; ++j) {
    const int vi = j * L + lir;
    if (!RAGGED || vbase + vi < NV) {
#pragma unroll
      for (int k = 0; k < V; ++k) lds[(vi * V + k) * P + rg] = src[j * V + k];
    }
  }
  __syncthreads();
  // a lane stores 16 bytes of a run: 4 floats, 8 bf16, 16 bytes of u8 (fewer where G does not divide)
  constexpr int WANT = 16 / (int)sizeof(typename fs_elem<DT>::type);
  constexpr int RUN = (G % WANT == 0) ? WANT : (G % 4 == 0) ? 4 : 1;
  constexpr int RPC = G / RUN;  // runs per output row
  const bool vec_ok = RUN > 1 && (R % RUN) == 0;
  const int col0 = vbase * V;
  for (int i = (int)threadIdx.x; i < TC * RPC; i += WG) {
    const int c = i / RPC, g0 = (i % RPC) * RUN;
    const long r = tile_row0 + g0;
    if (col0 + c >= CTOT) continue;
    float tmp[RUN];
#pragma unroll
    for (int q = 0; q < RUN; ++q) tmp[q] = lds[c * P + g0 + q];
    const long o = (long)(col0 + c) * R + r;
    if (RUN > 1 && vec_ok && r + RUN - 1 < R) {
      fs_store_vec<DT, RUN, NT>(tmp, base, o);
    } else {
#pragma unroll
      for (int q = 0; q < RUN; ++q)
        if (r + q < R) fs_store1_fwd<DT>(base, o + q, tmp[q]);
    }
  }
}

template <int DT> FS_DEV float fs_load1(const void* base, long i) {
  return fs_to_f32<DT>(static_cast<const typename fs_elem<DT>::type*>(base)[i]);
}
template <int DT> FS_DEV void fs_store1(void* base, long i, float x) {
  static_cast<typename fs_elem<DT>::type*>(base)[i] = fs_from_f32<DT>(x);
}

// ------------------------------------------------------------------------------------------
// reductions
// ------------------------------------------------------------------------------------------
template <int KIND> FS_DEV float fs_red_identity() {
  return KIND == FS_K_MAX ? -__builtin_inff() : KIND == FS_K_MIN ? __builtin_inff() : 0.0f;
}
template <int KIND> FS_DEV float fs_red_op(float a, float b) {
  return KIND == FS_K_MAX ? __builtin_fmaxf(a, b) : KIND == FS_K_MIN ? __builtin_fminf(a, b) : a + b;
}

// Serial reduction of the lane's own E elements (masked columns contribute the identity).
template <int KIND, int V, int NVL, int L, int NV, bool RAGGED>
FS_DEV float fs_lane_reduce(const float (&v)[NVL * V], int lir, int vbase = 0) {
  float acc = fs_red_identity<KIND>();
#pragma unroll
  for (int j = 0; j < NVL; ++j) {
    const bool ok = !RAGGED || (vbase + j * L + lir) < NV;
#pragma unroll
    for (int k = 0; k < V; ++k) acc = fs_red_op<KIND>(acc, ok ? v[j * V + k] : fs_red_identity<KIND>());
  }
  return acc;
}

template <int CTRL> FS_DEV float fs_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// DPP permute that only writes the rows of 16 lanes selected by ROW_MASK; the others receive `old`.
template <int CTRL, int ROW_MASK> FS_DEV float fs_dpp_rows(float old, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}

// All-reduce inside aligned segments of W lanes of a wavefront (W = 1,2,4,...,64).  Every
// lane of a segment ends with the same bits.  Steps 1..8 are DPP lane permutes inside a row
// of 16 lanes (quad_perm, row_half_mirror, row_mirror), fused into the arithmetic
// instruction.  Across the four rows of a whole wavefront two row broadcasts (lane 15 of a row
// into the next row, lane 31 into rows 2 and 3) leave the total in lane 63, which is read into a
// scalar register: (r3 op r2) op (r1 op r0), 6 permuting instructions and one v_readlane.  Two
// segments of 32 lanes read their row totals into scalar registers and fold them there.  No LDS
// traffic.
template <int KIND, int W> FS_DEV float fs_segment_allreduce(float v) {
  if constexpr (W >= 2) v = fs_red_op<KIND>(v, fs_dpp<0xB1>(v));   // quad_perm [1,0,3,2]
  if constexpr (W >= 4) v = fs_red_op<KIND>(v, fs_dpp<0x4E>(v));   // quad_perm [2,3,0,1]
  if constexpr (W >= 8) v = fs_red_op<KIND>(v, fs_dpp<0x141>(v));  // row_half_mirror
  if constexpr (W >= 16) v = fs_red_op<KIND>(v, fs_dpp<0x140>(v)); // row_mirror
  if constexpr (W >= 64) {
    const float idn = fs_red_identity<KIND>();                     // (what the rows left out by the mask combine with)
    v = fs_red_op<KIND>(v, fs_dpp_rows<0x142, 0xa>(idn, v));       // row_bcast:15 -> rows 1 and 3
    v = fs_red_op<KIND>(v, fs_dpp_rows<0x143, 0xc>(idn, v));       // row_bcast:31 -> rows 2 and 3
    v = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
  } else if constexpr (W >= 32) {
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    const float lo = fs_red_op<KIND>(r0, r1), hi = fs_red_op<KIND>(r2, r3);
    v = (__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) < 32u) ? lo : hi;
  }
  return v;
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads/stores of the
// streaming body are not waited for.
FS_DEV void fs_lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Cross-wave step of a row reduction when a row spans WPR = L/64 wavefronts: wave leaders
// publish their partial in LDS, one barrier, every lane folds the WPR partials in fixed order
// (so all lanes of the row hold identical bits).  `slot` points at this row-group's WPR*K
// floats inside the current ping-pong half; K reductions of one stage share the barrier.
template <int K, int WPR> struct fs_xwave {
  float* slot;
  int wir;     // wave index inside the row
  bool leader; // lane 0 of its wavefront
  FS_DEV void put(int k, float v) const {
    if (leader) slot[wir * K + k] = v;
  }
  template <int KIND> FS_DEV float get(int k) const {
    float acc = slot[k];
#pragma unroll
    for (int w = 1; w < WPR; ++w) acc = fs_red_op<KIND>(acc, slot[w * K + k]);
    return acc;
  }
};

// ------------------------------------------------------------------------------------------
// column reductions: two stages, no atomics on data, bitwise deterministic.
//   stage 1  every lane accumulates its columns over the rows its workgroup visits; the G
//            row-groups of the workgroup are folded through LDS in row-group order.
//   stage 2  the workgroup's partial goes to the workspace; a ticket per fan-in group tells
//            the last arriver to fold that group's partials in index order, and it moves up
//            one level.  The only atomic is the ticket.  The survivor of the top level holds
//            the result.
// The K column reductions of a kernel travel together as one vector of K*C floats, cut into
// chunks of FV floats (FV = 4 when C allows).  Thread t owns chunks t, t+WG, ...; chunk c
// belongs to reduction c / (C/FV) and covers columns (c % (C/FV))*FV onwards.
// ------------------------------------------------------------------------------------------
template <int K, int C, int WG, int FV> struct fs_colfold {
  static constexpr int CH = C / FV;                   // chunks per reduction
  static constexpr int NCH = K * CH;                  // chunks per workgroup partial
  static constexpr int CPT = (NCH + WG - 1) / WG;     // chunks per thread
};

// 4/8/16-byte memory access that is coherent at device scope without fences: the sc1 bit makes a
// store write through to, and a load read from, the level all 8 XCDs share.
typedef fs_u32 fs_u32x2 __attribute__((ext_vector_type(2)));
typedef fs_u32 fs_u32x4 __attribute__((ext_vector_type(4)));
#define FS_AUX_SC1 0x10
FS_DEV __amdgpu_buffer_rsrc_t fs_make_rsrc(const void* base, fs_u32 bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
template <int FV> FS_DEV void fs_load_dev(float (&dst)[FV], __amdgpu_buffer_rsrc_t r, fs_u32 byte_off) {
  if constexpr (FV == 4) {
    // (each element is copied to a scalar first: a bit_cast applied directly to a vector
    // element expression reads element 0 with this compiler)
    const fs_u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, FS_AUX_SC1);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      const fs_u32 w = u[f];
      dst[f] = __builtin_bit_cast(float, w);
    }
  } else if constexpr (FV == 2) {
    const fs_u32x2 u = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, FS_AUX_SC1);
    const fs_u32 w0 = u[0], w1 = u[1];
    dst[0] = __builtin_bit_cast(float, w0);
    dst[1] = __builtin_bit_cast(float, w1);
  } else {
    dst[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, FS_AUX_SC1));
  }
}
template <int FV> FS_DEV void fs_store_dev(const float (&src)[FV], __amdgpu_buffer_rsrc_t r, fs_u32 byte_off) {
  if constexpr (FV == 4) {
    fs_u32x4 u;
#pragma unroll
    for (int f = 0; f < 4; ++f) u[f] = __builtin_bit_cast(fs_u32, src[f]);
    __builtin_amdgcn_raw_buffer_store_b128(u, r, byte_off, 0, FS_AUX_SC1);
  } else if constexpr (FV == 2) {
    fs_u32x2 u;
    u[0] = __builtin_bit_cast(fs_u32, src[0]);
    u[1] = __builtin_bit_cast(fs_u32, src[1]);
    __builtin_amdgcn_raw_buffer_store_b64(u, r, byte_off, 0, FS_AUX_SC1);
  } else {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(fs_u32, src[0]), r, byte_off, 0, FS_AUX_SC1);
  }
}

FS_DEV int fs_lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }
// value of lane (lane ^ mask) of the same wavefront (LDS crossbar, no LDS memory)
FS_DEV float fs_shfl_xor(float v, int mask) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((fs_lane_id() ^ mask) << 2, __builtin_bit_cast(int, v)));
}

// Stage 1, in-workgroup fold of reduction number KIDX.  acc: the lane's per-column accumulators
// in the row layout.  Fills the chunks of `vals` that belong to reduction KIDX.  When several
// row-groups share a wavefront (L < 64) they are folded inside the wavefront first (lanes l,
// l+L, l+2L, ... own the same columns), so the LDS area holds one row per wavefront (GL = WG/64
// rows), not one per row-group.  The C columns go through the area PC columns at a time (PC a
// multiple of 8, or C itself): wide rows need no more LDS than narrow ones, only more barriers.
template <int KIND, int KIDX, int K, int V, int NVL, int L, int NV, int C, int WG, int FV, int PC, int CPT>
FS_DEV void fs_colred_fold_wg(const float (&acc_in)[NVL * V], float (&vals)[CPT][FV], float* lds /* GL*PC floats */, int lir, int rg) {
  typedef fs_colfold<K, C, WG, FV> S;
  static_assert(CPT == S::CPT, "chunks per thread");
  static_assert(PC == C || PC % 8 == 0, "piece width");
  constexpr int GL = L < 64 ? WG / 64 : WG / L;
  float acc[NVL * V];
#pragma unroll
  for (int e = 0; e < NVL * V; ++e) acc[e] = acc_in[e];
  if constexpr (L < 64) {
#pragma unroll
    for (int m = L; m < 64; m <<= 1) {
#pragma unroll
      for (int e = 0; e < NVL * V; ++e) {
        const float other = fs_shfl_xor(acc[e], m);
        // both partners compute op(lower, upper): identical bits in both
        const bool upper = (fs_lane_id() & m) != 0;
        acc[e] = fs_red_op<KIND>(upper ? other : acc[e], upper ? acc[e] : other);
      }
    }
  }
  const int slot = L < 64 ? (int)threadIdx.x / 64 : rg;
  const bool writer = L < 64 ? (fs_lane_id() < L) : true;
  if constexpr (PC >= C) {  // the whole row at once
    __syncthreads();  // the LDS area may still be read by the previous fold
    if (writer) {
#pragma unroll
      for (int j = 0; j < NVL; ++j) {
        const int vi = j * L + lir;
        if (vi < NV) {
#pragma unroll
          for (int k = 0; k < V; ++k) lds[slot * C + vi * V + k] = acc[j * V + k];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < S::CPT; ++i) {
      const int c = (int)threadIdx.x + i * WG;
      if (c >= KIDX * S::CH && c < (KIDX + 1) * S::CH) {
        const int col0 = (c - KIDX * S::CH) * FV;
#pragma unroll
        for (int f = 0; f < FV; ++f) {
          float a = lds[col0 + f];
          for (int g = 1; g < GL; ++g) a = fs_red_op<KIND>(a, lds[g * C + col0 + f]);
          vals[i][f] = a;
        }
      }
    }
    return;
  }
  for (int p0 = 0; p0 < C; p0 += PC) {
    __syncthreads();  // the LDS area may still be read by the previous piece or fold
    if (writer) {
#pragma unroll
      for (int j = 0; j < NVL; ++j) {
        const int vi = j * L + lir, col = vi * V - p0;
        if (vi < NV && col >= 0 && col < PC) {
#pragma unroll
          for (int k = 0; k < V; ++k) lds[slot * PC + col + k] = acc[j * V + k];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < S::CPT; ++i) {
      const int c = (int)threadIdx.x + i * WG;
      const int col0 = (c - KIDX * S::CH) * FV - p0;
      if (c >= KIDX * S::CH && c < (KIDX + 1) * S::CH && col0 >= 0 && col0 < PC) {
#pragma unroll
        for (int f = 0; f < FV; ++f) {
          float a = lds[col0 + f];
          for (int g = 1; g < GL; ++g) a = fs_red_op<KIND>(a, lds[g * PC + col0 + f]);
          vals[i][f] = a;
        }
      }
    }
  }
}

// Stage 2, grid-wide fold with fan-in F.
//   part     workspace, sum over levels of n_level*K*C floats
//   tickets  workspace, one zero-initialised u32 per fan-in group per level; left zero on exit
//   flag     one u32 of LDS
//   idx, n   this workgroup's index among the n workgroups that fold together (the whole grid,
//            or the workgroups of one column tile)
// Returns true in exactly one workgroup, whose `vals` then hold the final values.
//
// Visibility across the 8 XCDs (each has its own L2) is obtained without device-scope fences,
// which write back and invalidate a whole L2 and cost microseconds each: partials are written
// with sc1 stores, every wavefront waits for its own stores to be acknowledged before the
// workgroup barrier, lane 0 then bumps the ticket with an agent-scope atomic, and the folding
// workgroup reads the partials with sc1 loads (never served by stale lines of its own L2).
// The F loads of a chunk are independent and issued in batches, so a fold costs a few memory
// round trips, not F of them; they are combined in index order, whichever workgroup folds.
template <int K, int C, int WG, int FV, int F, typename KINDS, int CPT>
FS_DEV bool fs_colred_fold_grid(float (&vals)[CPT][FV], float* part, fs_u32* tickets, fs_u32* flag, fs_u32 idx, fs_u32 n) {
  typedef fs_colfold<K, C, WG, FV> S;
  static_assert(CPT == S::CPT, "chunks per thread");
  constexpr int KC = K * C;
  constexpr int FB = 16;  // loads in flight per chunk
  const int t = (int)threadIdx.x;
  while (n > 1) {
    {
      const __amdgpu_buffer_rsrc_t mine = fs_make_rsrc(part + (long)idx * KC, KC * 4);
#pragma unroll
      for (int i = 0; i < S::CPT; ++i) {
        const int c = t + i * WG;
        if (c < S::NCH) fs_store_dev<FV>(vals[i], mine, (fs_u32)c * (FV * 4));
      }
    }
    __builtin_amdgcn_s_waitcnt(0);  // this wavefront's partial stores are acknowledged
    __syncthreads();
    const fs_u32 grp = idx / F, first = grp * F;
    const fs_u32 cnt = (n - first) < (fs_u32)F ? (n - first) : (fs_u32)F;
    if (t == 0) {
      const fs_u32 old = __hip_atomic_fetch_add(&tickets[grp], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const bool last = old == cnt - 1;
      if (last) __hip_atomic_store(&tickets[grp], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *flag = last ? 1u : 0u;
    }
    __syncthreads();
    if (*flag == 0u) return false;
    const __amdgpu_buffer_rsrc_t theirs = fs_make_rsrc(part + (long)first * KC, cnt * (KC * 4));
#pragma unroll
    for (int i = 0; i < S::CPT; ++i) {
      const int c = t + i * WG;
      if (c < S::NCH) {
        const int k = c / S::CH;
        float a[FV];
#pragma unroll
        for (int f = 0; f < FV; ++f) a[f] = KINDS::identity(k);
        for (fs_u32 jb = 0; jb < cnt; jb += FB) {
          float tmp[FB][FV];
#pragma unroll
          for (int u = 0; u < FB; ++u) {
            const fs_u32 j = (jb + u) < cnt ? (jb + u) : (cnt - 1);  // clamped: always a valid load
            fs_load_dev<FV>(tmp[u], theirs, j * (KC * 4) + (fs_u32)c * (FV * 4));
          }
#pragma unroll
          for (int u = 0; u < FB; ++u) {
            const bool use = (jb + u) < cnt;
#pragma unroll
            for (int f = 0; f < FV; ++f) a[f] = use ? KINDS::op(k, a[f], tmp[u][f]) : a[f];
          }
        }
#pragma unroll
        for (int f = 0; f < FV; ++f) vals[i][f] = a[f];
      }
    }
    part += (long)n * KC;
    const fs_u32 groups = (n + F - 1) / F;
    tickets += groups;
    idx = grp;
    n = groups;
  }
  return true;
}

#endif  // FS_DEVICE_H_
