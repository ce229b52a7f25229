// `windows` transformer (Table 1) as an explicit gather: out[a, p.., q..] = in[a, p_i*s_i+q_i-lo_i ..].
//
// windows_generic : any 1..4 compute dims, one output element per thread, consecutive threads
//                   write consecutive output elements (coalesced stores, cached gathers).
// windows_chw     : the convolution shape of Fig. 2a / Fig. 5 -- in ((N),(C,H,W)), window
//                   (C,Kh,Kw) -- whose output is the im2col matrix, one row of K = C*Kh*Kw
//                   elements per output position.  A workgroup owns one output row (n, x): it
//                   stages the C*Kh input rows that row needs in LDS (coalesced 16-byte reads,
//                   padding cells filled in), then emits the Wo matrix rows, which are contiguous
//                   in memory, as 16-byte stores whose elements are gathered from LDS through a
//                   small table k -> LDS offset of (c, dx, dy).  HBM sees every input row
//                   Kh/Sh times (served by L2: neighbouring rows run on the same XCD) and every
//                   output byte exactly once.
#include "common.h"

#include <array>
#include <map>
#include <mutex>

namespace gs {

template <typename T, typename IdxT>
__global__ void __launch_bounds__(256)
windows_generic_kernel(const T* __restrict__ in, T* __restrict__ out, WindowsArgs a, IdxT total,
                       IdxT win_elems, IdxT out_pos) {
  // total = outer * out_pos * win_elems logical output elements.
  for (IdxT f = IdxT(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += IdxT(gridDim.x) * blockDim.x) {
    IdxT q = f % win_elems;
    IdxT row = f / win_elems;          // (outer, p..) flattened
    IdxT p = row % out_pos;
    IdxT o = row / out_pos;
    int64_t src = o;
    bool inside = true;
    // Decode p and q from the innermost dim outwards, accumulating the source offset.
    int64_t off = 0, mul = 1;
    for (int d = a.n_compute - 1; d >= 0; --d) {
      IdxT qd = q % IdxT(a.win[d]);
      q /= IdxT(a.win[d]);
      IdxT pd = p % IdxT(a.out_dim[d]);
      p /= IdxT(a.out_dim[d]);
      int64_t pos = int64_t(pd) * a.stride[d] + int64_t(qd) - a.pad_lo[d];
      inside = inside && pos >= 0 && pos < a.in_dim[d];
      off += pos * mul;
      mul *= a.in_dim[d];
    }
    src = src * mul + off;
    T v;
    if (inside) {
      v = in[src];
    } else {
      uint32_t bits = a.fill_bits;
      v = *reinterpret_cast<const T*>(&bits);
    }
    out[int64_t(row) * a.out_row_stride + int64_t(f % win_elems)] = v;
  }
}

// Pad columns [K, out_row_stride) of every row with zeros (only used when the row stride is padded).
template <typename T>
__global__ void __launch_bounds__(256)
windows_pad_tail_kernel(T* __restrict__ out, int64_t rows, int64_t K, int64_t ld) {
  const int64_t tail = ld - K;
  const int64_t total = rows * tail;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    out[(f / tail) * ld + K + (f % tail)] = T(0);
  }
}

template <typename T>
static hipError_t launch_generic_t(const WindowsArgs& a, hipStream_t s) {
  int64_t win_elems = 1, out_pos = 1;
  for (int d = 0; d < a.n_compute; ++d) {
    win_elems *= a.win[d];
    out_pos *= a.out_dim[d];
  }
  const int64_t total = a.outer * out_pos * win_elems;
  if (total == 0) return hipSuccess;
  const int threads = 256;
  const int64_t blocks64 = ceil_div(total, threads);
  const int blocks = int(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
  if (total < (int64_t(1) << 31)) {
    hipLaunchKernelGGL((windows_generic_kernel<T, uint32_t>), dim3(blocks), dim3(threads), 0, s,
                       static_cast<const T*>(a.in), static_cast<T*>(a.out), a, uint32_t(total),
                       uint32_t(win_elems), uint32_t(out_pos));
  } else {
    hipLaunchKernelGGL((windows_generic_kernel<T, int64_t>), dim3(blocks), dim3(threads), 0, s,
                       static_cast<const T*>(a.in), static_cast<T*>(a.out), a, total, win_elems,
                       out_pos);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.out_row_stride > win_elems) {
    const int64_t rows = a.outer * out_pos;
    const int64_t t2 = rows * (a.out_row_stride - win_elems);
    const int64_t b2 = ceil_div(t2, threads);
    hipLaunchKernelGGL((windows_pad_tail_kernel<T>), dim3(int(b2 < (1 << 20) ? b2 : (1 << 20))),
                       dim3(threads), 0, s, static_cast<T*>(a.out), rows, win_elems,
                       a.out_row_stride);
    e = hipGetLastError();
  }
  return e;
}

// ---------------------------------------------------------------------------------------------
// Convolution-shaped windows through LDS.
// ---------------------------------------------------------------------------------------------
struct WindowsChwArgs {
  const void* in;
  void* out;
  int N, C, H, W, Ho, Wo, Kh, Kw, Sh, Sw, Ph, Pw;
  int K;          // C*Kh*Kw
  int ld;         // elements between matrix rows (>= K; columns K..ld are written as zeros)
  int CC;         // channels staged per pass
  int pitch;      // LDS row pitch in elements (a whole number of dwords)
  int XO;         // first data column of an LDS row (left halo before it)
  int total;      // N*Ho workgroup tasks
  int per_xcd;    // tasks per XCD (ceil(total / 8))
  uint32_t fill_bits;
  int vec_ok;     // input rows are whole VB-byte vectors: staged through register prefetch
  FastDiv dvpr, dW, dhalo, dKh, dT, dKw;
};

constexpr int kChwLdsBudget = 40 * 1024;
constexpr int kStageBatch = 10;     // most 16-byte loads a thread keeps in flight while staging
constexpr int kChwPitchSlack = 8;    // dwords the pitch search may add to a row

// A workgroup walks over (task, channel pass) units.  While it emits one unit out of LDS, the
// 16-byte global loads of the next unit are already in flight into registers, so the memory
// latency of staging overlaps the emit phase instead of preceding it.
template <typename T, int B, int VB>   // a thread stages up to B vectors of VB (16, 8 or 4) bytes per unit
__global__ void __launch_bounds__(256)
windows_chw_kernel(WindowsChwArgs a) {
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;           // elements per 16-byte store
  typedef uint32_t tabv_t __attribute__((ext_vector_type(EPV)));
  typedef T outv_t __attribute__((ext_vector_type(EPV)));
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
  const int tid = threadIdx.x;
  // Workgroup i runs on XCD i % 8.  Each XCD takes a contiguous range of tasks and its
  // workgroups walk that range together, so tasks that share input rows meet in one L2.
  const int xcd = int(blockIdx.x % 8), lane_wg = int(blockIdx.x / 8), wgs = int(gridDim.x / 8);
  const int T_ = a.Kh * a.Kw;
  const int npass = (a.C + a.CC - 1) / a.CC;
  const int rows_max = a.CC * a.Kh + 1;                 // + one row of zeros for the pad columns
  const int row_bytes = a.pitch * ESZ;
  T* stage = reinterpret_cast<T*>(lds_raw);
  uint32_t* tab = reinterpret_cast<uint32_t*>(lds_raw + round_up(int64_t(rows_max) * row_bytes, 16));
  const T* in = static_cast<const T*>(a.in);
  T fill;
  {
    const uint32_t bits = a.fill_bits;
    fill = *reinterpret_cast<const T*>(&bits);
  }
  outv_t fv;
#pragma unroll
  for (int i = 0; i < EPV; ++i) fv[i] = fill;
  const bool vec_ok = a.vec_ok != 0;
  const int vpr = a.W * ESZ / VB;                       // vectors per input row
  constexpr int VD = VB / 4;                            // dwords per vector
  constexpr int EPL = VB / ESZ;                         // elements per vector
  typedef int32_t ldv_t __attribute__((ext_vector_type(VD)));
  const int halo = a.pitch - a.W;                       // cells of an LDS row outside the data
  const int zero_row = (rows_max - 1) * a.pitch;

  auto task_valid = [&](int tl) { return tl < a.per_xcd && xcd * a.per_xcd + tl < a.total; };

  // Registers of the unit being fetched: up to B vectors per thread.
  ldv_t val[B];
  ldv_t fillv;
#pragma unroll
  for (int i = 0; i < VD; ++i) fillv[i] = __builtin_bit_cast(i32x4, fv)[i];
  auto issue_loads = [&](int tl, int pass) {
    const int task = xcd * a.per_xcd + tl;
    const int n = task / a.Ho, ho = task - n * a.Ho;
    const int c0 = pass * a.CC;
    const int cc = a.C - c0 < a.CC ? a.C - c0 : a.CC;
    const int nvec = cc * a.Kh * vpr;
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int id = u * 256 + tid;
      uint32_t r, v, c, dx;
      a.dvpr.divmod(uint32_t(id), &r, &v);
      a.dKh.divmod(r, &c, &dx);
      const int ih = ho * a.Sh + int(dx) - a.Ph;
      val[u] = fillv;
      if (id < nvec && ih >= 0 && ih < a.H)
        val[u] = *reinterpret_cast<const ldv_t*>(
            in + ((int64_t(n) * a.C + c0 + int(c)) * a.H + ih) * a.W + int(v) * EPL);
    }
  };
  auto build_table = [&](int c0, int kbase, int nchunk) {
    // matrix column k -> LDS byte offset of (c, dx, dy) for output column 0
    for (int id = tid; id < nchunk * EPV; id += 256) {
      const int k = kbase + id;
      int off = zero_row;
      if (k < a.K) {
        uint32_t c, t, dx, dy;
        a.dT.divmod(uint32_t(k), &c, &t);
        a.dKw.divmod(t, &dx, &dy);
        off = ((int(c) - c0) * a.Kh + int(dx)) * a.pitch + a.XO - a.Pw + int(dy);
      }
      tab[id] = uint32_t(off * ESZ);
    }
  };

  int tl = lane_wg, pass = 0;
  if (!task_valid(tl)) return;
  // Written once: padding cells of every row, the row of zeros, and (single pass) the table.
  for (int id = tid; id < (rows_max - 1) * halo; id += 256) {
    uint32_t r, h;
    a.dhalo.divmod(uint32_t(id), &r, &h);
    stage[int(r) * a.pitch + (int(h) < a.XO ? int(h) : a.W + int(h))] = fill;
  }
  for (int id = tid; id < a.pitch; id += 256) stage[zero_row + id] = T(0);
  if (npass == 1) build_table(0, 0, a.ld / EPV);
  if (vec_ok) issue_loads(tl, pass);

  while (task_valid(tl)) {
    const int task = xcd * a.per_xcd + tl;
    const int n = task / a.Ho, ho = task - n * a.Ho;
    const int c0 = pass * a.CC;
    const int cc = a.C - c0 < a.CC ? a.C - c0 : a.CC;
    const bool last = c0 + cc >= a.C;
    const int nrows = cc * a.Kh;
    const int kbase = c0 * T_;
    const int kend = last ? a.ld : (c0 + cc) * T_;      // the last pass also writes the pad columns
    const int nchunk = (kend - kbase) / EPV;
    T* out = static_cast<T*>(a.out) + (int64_t(n) * a.Ho + ho) * a.Wo * int64_t(a.ld);
    __syncthreads();                                    // the previous unit has finished reading
    // -- stage the input rows (c, dx): image row ho*Sh + dx - Ph of channel c0 + c.  LDS rows
    //    start on dword, not 16-byte, boundaries (the pitch is chosen against bank conflicts).
    if (vec_ok) {
      const int nvec = nrows * vpr;
#pragma unroll
      for (int u = 0; u < B; ++u) {
        const int id = u * 256 + tid;
        if (id < nvec) {
          uint32_t r, v;
          a.dvpr.divmod(uint32_t(id), &r, &v);
          int32_t* d = reinterpret_cast<int32_t*>(lds_raw + (int(r) * a.pitch + a.XO) * ESZ + int(v) * VB);
#pragma unroll
          for (int i = 0; i < VD; ++i) d[i] = val[u][i];
        }
      }
    } else {
      for (int id = tid; id < nrows * a.W; id += 256) {
        uint32_t r, x, c, dx;
        a.dW.divmod(uint32_t(id), &r, &x);
        a.dKh.divmod(r, &c, &dx);
        const int ih = ho * a.Sh + int(dx) - a.Ph;
        stage[int(r) * a.pitch + a.XO + int(x)] =
            (ih >= 0 && ih < a.H) ? in[((int64_t(n) * a.C + c0 + int(c)) * a.H + ih) * a.W + int(x)] : fill;
      }
    }
    if (npass > 1) build_table(c0, kbase, nchunk);
    __syncthreads();
    // -- next unit: its loads fly while this one is emitted
    int ntl = tl, npass_i = pass + 1;
    if (npass_i == npass) {
      npass_i = 0;
      ntl += wgs;
    }
    if (vec_ok && task_valid(ntl)) issue_loads(ntl, npass_i);
    // -- emit: item = (output column y, 16-byte chunk j of the k range of this pass); a thread
    //    takes items tid, tid + 256, ...; (y, j) advance without dividing again.
    const int items = a.Wo * nchunk;
    const int my_items = items > tid ? (items - tid + 255) / 256 : 0;
    const int step_y = 256 / nchunk, step_j = 256 - step_y * nchunk;
    int y = tid / nchunk, j = tid - y * nchunk;
#pragma unroll 2
    for (int it = 0; it < my_items; ++it) {
      const tabv_t offs = *reinterpret_cast<const tabv_t*>(tab + j * EPV);
      const uint32_t shift = uint32_t(y * a.Sw * ESZ);
      outv_t v;
#pragma unroll
      for (int i = 0; i < EPV; ++i) v[i] = *reinterpret_cast<const T*>(lds_raw + (offs[i] + shift));
      // written once, never read back by this kernel: keep it from displacing the input rows in L2
      __builtin_nontemporal_store(v, reinterpret_cast<outv_t*>(out + int64_t(y) * a.ld + kbase + j * EPV));
      j += step_j;
      y += step_y;
      if (j >= nchunk) {
        j -= nchunk;
        ++y;
      }
    }
    tl = ntl;
    pass = npass_i;
  }
}

// LDS bank-conflict cost of the emit phase's element reads for row pitch `pitch` (elements): for
// the first 128 lanes (two waves) and every element slot of a 16-byte chunk, lanes are served in
// groups of 32 and a group costs as many cycles as the fullest bank holds distinct dwords.
// Evaluated for 32 and for 64 banks; the sum ranks the candidates.
static int chw_conflict_cost(const WindowsChwArgs& a, int esz, int epv, int pitch, int nchunk) {
  int cost = 0;
  const int T_ = a.Kh * a.Kw;
  for (int banks = 32; banks <= 64; banks *= 2) {
    for (int i = 0; i < epv; ++i) {
      for (int g = 0; g < 4; ++g) {
        int64_t seen[64][8];
        int cnt[64] = {0};
        int worst = 0;
        for (int l = 0; l < 32; ++l) {
          const int id = g * 32 + l;
          const int y = id / nchunk, j = id % nchunk;
          if (y >= a.Wo) continue;
          const int k = j * epv + i;
          if (k >= a.K) continue;
          const int c = k / T_, t = k % T_;
          const int64_t byte = (int64_t(c * a.Kh + t / a.Kw) * pitch + a.XO - a.Pw + t % a.Kw +
                                int64_t(y) * a.Sw) * esz;
          const int64_t dw = byte / 4;
          const int b = int(dw % banks);
          bool dup = false;
          for (int q = 0; q < cnt[b] && q < 8; ++q) dup = dup || seen[b][q] == dw;
          if (!dup) {
            if (cnt[b] < 8) seen[b][cnt[b]] = dw;
            ++cnt[b];
          }
          if (cnt[b] > worst) worst = cnt[b];
        }
        cost += worst;
      }
    }
  }
  return cost;
}

static int chw_num_cus() {
  static int cus = 0;
  if (!cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

// Tries the LDS-staged kernel; returns hipErrorInvalidValue if the shape does not qualify.
template <typename T>
static hipError_t launch_chw_t(const WindowsArgs& w, hipStream_t s) {
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  constexpr int EPD = 4 / ESZ;            // elements per dword
  if (w.n_compute != 3 || w.win[0] != w.in_dim[0] || w.pad_lo[0] != 0 || w.out_dim[0] != 1)
    return hipErrorInvalidValue;
  for (int d = 0; d < 3; ++d)
    if (w.in_dim[d] > (1 << 20) || w.out_dim[d] > (1 << 20) || w.win[d] > (1 << 12) ||
        w.stride[d] > (1 << 12) || w.pad_lo[d] > (1 << 12))
      return hipErrorInvalidValue;
  WindowsChwArgs a;
  a.in = w.in;
  a.out = w.out;
  a.C = int(w.in_dim[0]); a.H = int(w.in_dim[1]); a.W = int(w.in_dim[2]);
  a.Ho = int(w.out_dim[1]); a.Wo = int(w.out_dim[2]);
  a.Kh = int(w.win[1]); a.Kw = int(w.win[2]);
  a.Sh = int(w.stride[1]); a.Sw = int(w.stride[2]);
  a.Ph = int(w.pad_lo[1]); a.Pw = int(w.pad_lo[2]);
  a.fill_bits = w.fill_bits;
  const int64_t K = int64_t(a.C) * a.Kh * a.Kw;
  const int64_t tasks = w.outer * a.Ho;
  if (K > (1 << 24) || tasks > (1 << 28) || w.outer > (1 << 24)) return hipErrorInvalidValue;
  if (w.out_row_stride > (1 << 24)) return hipErrorInvalidValue;
  a.N = int(w.outer);
  a.K = int(K);
  a.ld = int(w.out_row_stride);
  if ((int64_t(a.ld) * ESZ) % 16 != 0 || reinterpret_cast<uintptr_t>(w.out) % 16 != 0)
    return hipErrorInvalidValue;
  a.total = int(tasks);
  a.per_xcd = int(ceil_div(tasks, 8));
  if (a.total == 0 || a.Wo == 0 || a.ld == 0 || a.C == 0 || a.Kh == 0 || a.Kw == 0 || a.W == 0)
    return a.total == 0 || a.Wo == 0 || a.ld == 0 ? hipSuccess : hipErrorInvalidValue;
  a.XO = int(round_up(a.Pw, EPD));
  const int64_t reach = int64_t(a.XO) - a.Pw + int64_t(a.Wo - 1) * a.Sw + a.Kw;   // columns read
  const int64_t width = reach > a.XO + a.W ? reach : a.XO + a.W;
  const int base_pitch = int(round_up(width, EPD));
  const int max_pitch = base_pitch + kChwPitchSlack * EPD;
  // Channels per pass: as many as the LDS budget holds, in units that keep the k range of a pass
  // a whole number of 16-byte chunks.
  int unit = 1;
  while ((int64_t(unit) * a.Kh * a.Kw * ESZ) % 16 != 0) unit *= 2;
  auto bytes_for = [&](int cc, int pitch) {
    const int64_t tab_entries = round_up(int64_t(cc) * a.Kh * a.Kw + (a.ld - K), EPV) + EPV;
    return round_up((int64_t(cc) * a.Kh + 1) * pitch * ESZ, 16) + tab_entries * 4;
  };
  // Widest vector (16, 8 or 4 bytes) that input rows are whole numbers of and aligned to.
  int vb = 0;
  for (int cand = 16; cand >= 4 && !vb; cand /= 2)
    if ((a.W * ESZ) % cand == 0 && reinterpret_cast<uintptr_t>(w.in) % cand == 0) vb = cand;
  a.vec_ok = vb ? 1 : 0;
  const int64_t vpr = vb ? int64_t(a.W) * ESZ / vb : 1;
  const int maxb = kStageBatch;
  auto fits = [&](int c) {
    return bytes_for(c, max_pitch) <= kChwLdsBudget &&
           (!a.vec_ok || int64_t(c) * a.Kh * vpr <= 256 * maxb);   // one register batch per unit
  };
  int cc = a.C;
  if (!fits(cc)) {
    cc = int((kChwLdsBudget / (int64_t(a.Kh) * max_pitch * ESZ + int64_t(a.Kh) * a.Kw * 4)) / unit) * unit;
    if (cc > a.C) cc = a.C / unit * unit;
    while (cc >= unit && !fits(cc)) cc -= unit;
    if (cc < unit) return hipErrorInvalidValue;
  }
  a.CC = cc;
  // Pitch with the fewest bank conflicts for this shape, remembered per shape.
  {
    static std::mutex mu;
    static std::map<std::array<int, 12>, int> memo;
    const std::array<int, 12> key = {ESZ, a.C, a.W, a.Wo, a.Kh, a.Kw, a.Sw, a.Pw, a.ld, cc, a.K, base_pitch};
    std::lock_guard<std::mutex> lock(mu);
    auto it = memo.find(key);
    if (it == memo.end()) {
      const int nchunk = cc >= a.C ? a.ld / EPV : cc * a.Kh * a.Kw / EPV;
      int best = base_pitch, best_cost = 1 << 30;
      for (int p = base_pitch; p <= max_pitch; p += EPD) {
        const int cost = chw_conflict_cost(a, ESZ, EPV, p, nchunk);
        if (cost < best_cost) {
          best_cost = cost;
          best = p;
        }
      }
      it = memo.emplace(key, best).first;
    }
    a.pitch = it->second;
  }
  a.dvpr = FastDiv::make(uint32_t(vpr > 0 ? vpr : 1));
  a.dW = FastDiv::make(uint32_t(a.W));
  a.dhalo = FastDiv::make(uint32_t(a.pitch - a.W > 0 ? a.pitch - a.W : 1));
  a.dKh = FastDiv::make(uint32_t(a.Kh));
  a.dT = FastDiv::make(uint32_t(a.Kh * a.Kw));
  a.dKw = FastDiv::make(uint32_t(a.Kw));
  const size_t lds = size_t(bytes_for(cc, a.pitch));
  // Persistent workgroups: as many as fit the chip at once (by LDS), at most one per task.
  int per_cu = int((160 * 1024) / (lds + 512));
  per_cu = per_cu < 1 ? 1 : per_cu > 8 ? 8 : per_cu;
  // Tasks that each write a long run of matrix rows (tens of KB) go to at most two workgroups per
  // compute unit, several tasks each: fewer concurrent write streams measured 10 % faster (5.4
  // against 4.8 TB/s on the 3x3 workload); short tasks keep every workgroup that fits.
  if (int64_t(a.Wo) * a.ld * ESZ >= 16 * 1024 && per_cu > 2) per_cu = 2;
  int64_t wgs_per_xcd = int64_t(chw_num_cus()) * per_cu / 8;
  if (wgs_per_xcd > a.per_xcd) wgs_per_xcd = a.per_xcd;
  if (wgs_per_xcd < 1) wgs_per_xcd = 1;
  // Every workgroup gets the same number of tasks: as few workgroups as finish in that many rounds.
  wgs_per_xcd = ceil_div(a.per_xcd, ceil_div(a.per_xcd, wgs_per_xcd));
  const dim3 grid(unsigned(wgs_per_xcd) * 8);
  const int64_t need = a.vec_ok ? ceil_div(int64_t(cc) * a.Kh * vpr, 256) : 1;
#define GS_CHW_LAUNCH(VB_)                                                                            \
  {                                                                                                   \
    if (need <= 3) hipLaunchKernelGGL((windows_chw_kernel<T, 3, VB_>), grid, dim3(256), lds, s, a);   \
    else if (need <= 6) hipLaunchKernelGGL((windows_chw_kernel<T, 6, VB_>), grid, dim3(256), lds, s, a); \
    else hipLaunchKernelGGL((windows_chw_kernel<T, kStageBatch, VB_>), grid, dim3(256), lds, s, a);   \
  }
  if (vb == 8) GS_CHW_LAUNCH(8)
  else if (vb == 4) GS_CHW_LAUNCH(4)
  else GS_CHW_LAUNCH(16)
#undef GS_CHW_LAUNCH
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_windows_t(const WindowsArgs& a, hipStream_t s) {
  const hipError_t e = launch_chw_t<T>(a, s);
  if (e != hipErrorInvalidValue) return e;
  return launch_generic_t<T>(a, s);
}

hipError_t launch_windows(const WindowsArgs& a, hipStream_t s) {
  switch (a.esz) {
    case 1: return launch_windows_t<uint8_t>(a, s);
    case 2: return launch_windows_t<uint16_t>(a, s);
    case 4: return launch_windows_t<uint32_t>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace gs
