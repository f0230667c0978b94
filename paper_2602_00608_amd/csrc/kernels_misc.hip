// Small data-movement kernels: nearest-2x upsample, weight packing, strided
// transpose with type conversion (NCHW <-> NHWC, V -> V^T), fp32 copy.
#include "common.hpp"
#include "pack_layout.hpp"

namespace wmdec {
namespace {

struct alignas(16) Chunk16 { uint32_t w[4]; };

// y[n,oy,ox,:] = x[n,oy>>1,ox>>1,:] in 16-byte chunks (c*esize % 16 == 0): a thread reads one input chunk and
// writes it to the four output pixels it maps to, so the input is read exactly once and the index arithmetic is
// paid once per four stores.  A run of lanes covers whole pixels, i.e. every store instruction writes runs of
// cpp*16 contiguous bytes.
__global__ __launch_bounds__(256) void upsample2x_vec(const Chunk16* __restrict__ x, Chunk16* __restrict__ y,
                                                      int h_in, int w_in, int cpp /*chunks per pixel*/, size_t total_in) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total_in; i += (size_t)gridDim.x * 256) {
    const Chunk16 v = x[i];
    const int cc = (int)(i % cpp);
    size_t pix = i / cpp;
    const int ix = (int)(pix % w_in); pix /= w_in;
    const int iy = (int)(pix % h_in);
    const size_t n = pix / h_in;
    const size_t o = ((n * 2 * h_in + 2 * iy) * 2 * w_in + 2 * ix) * cpp + cc;
    const size_t row = (size_t)2 * w_in * cpp;
    y[o] = v; y[o + cpp] = v; y[o + row] = v; y[o + row + cpp] = v;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void upsample2x_elem(const T* __restrict__ x, T* __restrict__ y,
                                                       int h_in, int w_in, int c, size_t total) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int cc = (int)(i % c);
  size_t pix = i / c;
  const int ox = (int)(pix % (2 * w_in)); pix /= (2 * w_in);
  const int oy = (int)(pix % (2 * h_in));
  const size_t n = pix / (2 * h_in);
  y[i] = x[((n * h_in + (oy >> 1)) * w_in + (ox >> 1)) * c + cc];
}

// One thread per element of the packed destination (see pack_layout.hpp).  Rows [row_off, row_off+cout)
// of a destination with rows_total output channels are written from src[co][ci][tap]; padding elements
// (ci >= cin or row >= rows_total) are zeroed; rows that belong to another source are left alone.
template <typename S, typename D>
__global__ __launch_bounds__(256) void pack_conv_kernel(const S* __restrict__ src, D* __restrict__ dst, int cout, int cin,
                                                        int taps, int row_off, int rows_total) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int cinb = packed_cin_blocks(cin), coutb = packed_cout_blocks(rows_total);
  if (i >= (size_t)taps * cinb * coutb * 512) return;
  const int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  size_t blk = i >> 9;
  const int cob = (int)(blk % coutb); blk /= coutb;
  const int cib = (int)(blk % cinb);
  const int tap = (int)(blk / cinb);
  const int row = cob * 32 + (lane & 31), ci = cib * 16 + (lane >> 5) * 8 + e;
  if (ci >= cin || row >= rows_total) { dst[i] = from_float<D>(0.f); return; }
  const int co = row - row_off;
  if (co < 0 || co >= cout) return;
  dst[i] = from_float<D>(to_float(src[((size_t)co * cin + ci) * taps + tap]));
}

// Phase pack of a nearest-2x-upsample + 3x3 convolution.  Output pixel (2i + py, 2j + px) only sees input rows
// i + py - 1, i + py and columns j + px - 1, j + px; the 3x3 taps that fall on the same input pixel are summed once,
// here (fp32, fixed order, one rounding to D).  Row r of phase py collects ky in {0} | {1,2} (py = 0) or {0,1} | {2}
// (py = 1), the same for columns.  Tap index of the pack: ((py*2 + px)*2 + r)*2 + s, 16 taps.
template <typename S, typename D>
__global__ __launch_bounds__(256) void pack_upconv_phase_kernel(const S* __restrict__ src, D* __restrict__ dst, int cout, int cin) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int cinb = packed_cin_blocks(cin), coutb = packed_cout_blocks(cout);
  if (i >= (size_t)16 * cinb * coutb * 512) return;
  const int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
  size_t blk = i >> 9;
  const int cob = (int)(blk % coutb); blk /= coutb;
  const int cib = (int)(blk % cinb);
  const int tap = (int)(blk / cinb);
  const int co = cob * 32 + (lane & 31), ci = cib * 16 + (lane >> 5) * 8 + e;
  if (ci >= cin || co >= cout) { dst[i] = from_float<D>(0.f); return; }
  const int py = tap >> 3, px = (tap >> 2) & 1, r = (tap >> 1) & 1, sx = tap & 1;
  const int ky0 = py == 0 ? (r == 0 ? 0 : 1) : (r == 0 ? 0 : 2), ky1 = py == 0 ? (r == 0 ? 0 : 2) : (r == 0 ? 1 : 2);
  const int kx0 = px == 0 ? (sx == 0 ? 0 : 1) : (sx == 0 ? 0 : 2), kx1 = px == 0 ? (sx == 0 ? 0 : 2) : (sx == 0 ? 1 : 2);
  float acc = 0.f;
  for (int ky = ky0; ky <= ky1; ++ky)
    for (int kx = kx0; kx <= kx1; ++kx) acc += to_float(src[((size_t)co * cin + ci) * 9 + ky * 3 + kx]);
  dst[i] = from_float<D>(acc);
}

// dst[b][i][j] = src[b][j][i], 32x32 tiles through LDS.  BLOCKED (dst_ld = 0): the destination is cut into blocks of 32
// source rows, dst[b][j / 32][i][40] with j % 32 in the first 32 of a row's 40 elements and zeros for source rows past
// the end: the image of the attention kernel's V^T tile in LDS (32 keys, rows padded to 40 elements), which that
// kernel copies as one contiguous run.
template <typename S, typename D, bool BLOCKED = false>
__global__ __launch_bounds__(256) void transpose_kernel(const S* __restrict__ src, D* __restrict__ dst, int rows, int cols,
                                                        size_t src_ld, size_t src_bs, size_t dst_ld, size_t dst_bs) {
  __shared__ float tile[32][33];
  const int b = blockIdx.z;
  const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int k = ty; k < 32; k += 8) {
    const int r = r0 + k, c = c0 + tx;
    if (r < rows && c < cols) tile[k][tx] = to_float(src[(size_t)b * src_bs + (size_t)r * src_ld + c]);
  }
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int c = c0 + k, r = r0 + tx;
    if (BLOCKED) {
      if (c < cols) dst[(size_t)b * dst_bs + ((size_t)blockIdx.y * cols + c) * 40 + tx] = from_float<D>(r < rows ? tile[tx][k] : 0.f);
    } else if (r < rows && c < cols) {
      dst[(size_t)b * dst_bs + (size_t)c * dst_ld + r] = from_float<D>(tile[tx][k]);
    }
  }
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = src[i];
}

// plain copy, 16 bytes per thread: a kernel of known traffic that hardware counter passes are scaled by
__global__ __launch_bounds__(256) void copy_u128_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = src[i];
}

// one first-order extrapolation step count folded into `scale`: out = z + scale * v (Alg. 2, hit branch)
template <typename S, typename D>
__global__ __launch_bounds__(256) void axpy_kernel(const S* __restrict__ z, const S* __restrict__ v, float scale,
                                                   D* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) out[i] = from_float<D>(fmaf(scale, to_float(v[i]), to_float(z[i])));
}

template <typename S>
int axpy_s(const void* z, const void* v, float scale, void* out, int out_dtype, size_t count, hipStream_t s) {
  const dim3 grid((unsigned)((count + 255) / 256));
  switch (out_dtype) {
    case WMDEC_F32: hipLaunchKernelGGL((axpy_kernel<S, float>), grid, dim3(256), 0, s, (const S*)z, (const S*)v, scale, (float*)out, count); break;
    case WMDEC_BF16: hipLaunchKernelGGL((axpy_kernel<S, bf16_t>), grid, dim3(256), 0, s, (const S*)z, (const S*)v, scale, (bf16_t*)out, count); break;
    default: hipLaunchKernelGGL((axpy_kernel<S, f16_t>), grid, dim3(256), 0, s, (const S*)z, (const S*)v, scale, (f16_t*)out, count); break;
  }
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename S, typename D>
int pack_t(const void* src, void* dst, int cout, int cin, int k, int row_off, int rows_total, hipStream_t s) {
  const size_t total = packed_elems(k * k, rows_total, cin);
  hipLaunchKernelGGL((pack_conv_kernel<S, D>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                     (const S*)src, (D*)dst, cout, cin, k * k, row_off, rows_total);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename S, typename D>
int pack_phase_t(const void* src, void* dst, int cout, int cin, hipStream_t s) {
  const size_t total = packed_elems(16, cout, cin);
  hipLaunchKernelGGL((pack_upconv_phase_kernel<S, D>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                     (const S*)src, (D*)dst, cout, cin);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename S, typename D>
int transpose_t(const void* src, void* dst, int batch, int rows, int cols, size_t sld, size_t sbs, size_t dld, size_t dbs, hipStream_t s) {
  dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32), (unsigned)batch);
  if (dld == 0) hipLaunchKernelGGL((transpose_kernel<S, D, true>), grid, dim3(256), 0, s, (const S*)src, (D*)dst, rows, cols, sld, sbs, dld, dbs);
  else hipLaunchKernelGGL((transpose_kernel<S, D>), grid, dim3(256), 0, s, (const S*)src, (D*)dst, rows, cols, sld, sbs, dld, dbs);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

template <typename S>
int transpose_s(const void* src, void* dst, int dd, int batch, int rows, int cols, size_t sld, size_t sbs, size_t dld, size_t dbs, hipStream_t s) {
  switch (dd) {
    case WMDEC_F32: return transpose_t<S, float>(src, dst, batch, rows, cols, sld, sbs, dld, dbs, s);
    case WMDEC_BF16: return transpose_t<S, bf16_t>(src, dst, batch, rows, cols, sld, sbs, dld, dbs, s);
    default: return transpose_t<S, f16_t>(src, dst, batch, rows, cols, sld, sbs, dld, dbs, s);
  }
}

}  // namespace

int launch_upsample2x(const void* x, void* y, int dtype, int n, int h_in, int w_in, int c, hipStream_t s) {
  const size_t es = dtype_size(dtype);
  const size_t out_elems = (size_t)n * 4 * h_in * w_in * c;
  if (((size_t)c * es) % 16 == 0) {
    const int cpp = (int)((size_t)c * es / 16);
    const size_t total_in = out_elems / 4 * es / 16;
    size_t blocks = (total_in + 255) / 256;
    if (blocks > 8192) blocks = 8192;   // grid-stride beyond 32 workgroups per compute unit
    hipLaunchKernelGGL(upsample2x_vec, dim3((unsigned)blocks), dim3(256), 0, s,
                       (const Chunk16*)x, (Chunk16*)y, h_in, w_in, cpp, total_in);
  } else if (es == 4) {
    hipLaunchKernelGGL(upsample2x_elem<uint32_t>, dim3((unsigned)((out_elems + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)x, (uint32_t*)y, h_in, w_in, c, out_elems);
  } else {
    hipLaunchKernelGGL(upsample2x_elem<uint16_t>, dim3((unsigned)((out_elems + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)x, (uint16_t*)y, h_in, w_in, c, out_elems);
  }
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

int launch_pack_conv(const void* src, int src_dtype, int cout, int cin, int k, void* dst, int op_dtype,
                     int dst_row_offset, int dst_rows_total, hipStream_t s) {
  if (src_dtype == WMDEC_F32) {
    switch (op_dtype) {
      case WMDEC_F32: return pack_t<float, float>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
      case WMDEC_BF16: return pack_t<float, bf16_t>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
      default: return pack_t<float, f16_t>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
    }
  }
  switch (op_dtype) {
    case WMDEC_F32: return pack_t<bf16_t, float>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
    case WMDEC_BF16: return pack_t<bf16_t, bf16_t>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
    default: return pack_t<bf16_t, f16_t>(src, dst, cout, cin, k, dst_row_offset, dst_rows_total, s);
  }
}

size_t upconv_phase_offset_bytes(int cout, int cin, int op_dtype) { return packed_elems(9, cout, cin) * dtype_size(op_dtype); }
size_t upconv_packed_bytes(int cout, int cin, int op_dtype) { return packed_elems(9 + 16, cout, cin) * dtype_size(op_dtype); }

int launch_pack_upconv(const void* src, int src_dtype, int cout, int cin, void* dst, int op_dtype, hipStream_t s) {
  const int rc = launch_pack_conv(src, src_dtype, cout, cin, 3, dst, op_dtype, 0, cout, s);
  if (rc != WMDEC_OK) return rc;
  void* ph = (char*)dst + upconv_phase_offset_bytes(cout, cin, op_dtype);
  if (src_dtype == WMDEC_F32) {
    switch (op_dtype) {
      case WMDEC_F32: return pack_phase_t<float, float>(src, ph, cout, cin, s);
      case WMDEC_BF16: return pack_phase_t<float, bf16_t>(src, ph, cout, cin, s);
      default: return pack_phase_t<float, f16_t>(src, ph, cout, cin, s);
    }
  }
  switch (op_dtype) {
    case WMDEC_F32: return pack_phase_t<bf16_t, float>(src, ph, cout, cin, s);
    case WMDEC_BF16: return pack_phase_t<bf16_t, bf16_t>(src, ph, cout, cin, s);
    default: return pack_phase_t<bf16_t, f16_t>(src, ph, cout, cin, s);
  }
}

int launch_transpose(const void* src, int src_dtype, void* dst, int dst_dtype, int batch, int rows, int cols,
                     size_t src_ld, size_t src_batch_stride, size_t dst_ld, size_t dst_batch_stride, hipStream_t s) {
  switch (src_dtype) {
    case WMDEC_F32: return transpose_s<float>(src, dst, dst_dtype, batch, rows, cols, src_ld, src_batch_stride, dst_ld, dst_batch_stride, s);
    case WMDEC_BF16: return transpose_s<bf16_t>(src, dst, dst_dtype, batch, rows, cols, src_ld, src_batch_stride, dst_ld, dst_batch_stride, s);
    default: return transpose_s<f16_t>(src, dst, dst_dtype, batch, rows, cols, src_ld, src_batch_stride, dst_ld, dst_batch_stride, s);
  }
}

int launch_axpy(const void* z, const void* v, int dtype, float scale, void* out, int out_dtype, size_t count, hipStream_t s) {
  switch (dtype) {
    case WMDEC_F32: return axpy_s<float>(z, v, scale, out, out_dtype, count, s);
    case WMDEC_BF16: return axpy_s<bf16_t>(z, v, scale, out, out_dtype, count, s);
    default: return axpy_s<f16_t>(z, v, scale, out, out_dtype, count, s);
  }
}

__global__ void zero_u32_kernel(unsigned* p, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = 0u;
}

int launch_zero_u32(void* p, int count, hipStream_t s) {
  hipLaunchKernelGGL(zero_u32_kernel, dim3((unsigned)((count + 63) / 64)), dim3(64), 0, s, (unsigned*)p, count);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

int launch_copy_u128(const void* src, void* dst, size_t bytes, hipStream_t s) {
  const size_t count = bytes / 16;
  if (count == 0) return WMDEC_OK;
  WMDEC_REQUIRE((count + 255) / 256 <= 0x7fffffffu, WMDEC_ERR_UNSUPPORTED, "copy: too many bytes for one launch");
  hipLaunchKernelGGL(copy_u128_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, count);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

int launch_copy_f32(const float* src, float* dst, size_t count, hipStream_t s) {
  if (count == 0) return WMDEC_OK;
  hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, src, dst, count);
  WMDEC_HIP(hipGetLastError());
  return WMDEC_OK;
}

}  // namespace wmdec
