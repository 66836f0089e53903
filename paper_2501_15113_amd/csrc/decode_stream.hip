// Decode attention over the ragged bf16 cache, balanced streaming form.
//
// The decode step must read every kept K and V row once; nothing else matters
// for its run time.  Measured on MI355X, HBM read bandwidth keeps rising with
// the number of bytes in flight (about 6.2 TB/s at 256 KB per CU, 7 TB/s at
// 512 KB per CU), and a kernel whose workgroups finish at different times
// loses the tail.  Hence:
//
//   * the unit of work is the 32-token page; the T pages a step must read are
//     dealt out evenly, wave i of W takes pages [i*T/W, (i+1)*T/W) of the
//     concatenated page list of all units, so all waves finish together
//     whatever the mix of 131072-token and 1028-token units is;
//   * every wave keeps a ring of NP pages (16 KB each) in flight in its
//     registers -- the VGPR file is the largest landing zone on the CU;
//   * a wave whose range crosses unit boundaries writes one online-softmax
//     partial (m, l, o) per unit it touched, slot = wave + unit, which is unique
//     because both indices only grow along the page list; the combine kernel
//     merges the slots of a unit in ascending order.
//
// Waves never synchronise with each other after the prologue.
#include "decode_common.h"

namespace taskkv {

constexpr int MAXU = STREAM_MAX_UNITS;

// First page of wave i when T pages are dealt to W waves.  Workgroups go to
// the eight XCDs round robin, and under a saturating read stream the odd XCDs
// of this part deliver about a tenth less bandwidth than their even
// neighbours (measured on every launch and every allocation), so with equal
// ranges the even half of the chip idles while the odd half finishes.  The
// waves of even workgroups therefore take (1024 + skew) / 1024 of an equal
// share and those of odd workgroups (1024 - skew) / 1024; a pair of workgroups
// (eight waves) always covers eight equal shares.  W is a multiple of 8
// whenever skew != 0.
__device__ __forceinline__ int64_t range_start(int i, int64_t T, int W, int skew) {
  const int r = i & 7;
  const int64_t c = (int64_t)(i - r) * 1024 +
                    (r <= 4 ? r * (1024 + skew) : 4 * (1024 + skew) + (r - 4) * (1024 - skew));
  // c T < 2^53 and the quotient, when it is not an integer, lies at least
  // 1 / (1024 W) from the next one: the correctly rounded fp64 quotient has the
  // same floor as the 64-bit integer division, which costs a wave ten times as
  // many instructions at the head of every launch
  return (int64_t)((double)c * (double)T / ((double)W * 1024.0));
}
// What the decode kernel leaves behind for the combine kernel, after the
// units + 1 page prefixes: the first page of every wave's range (W + 1
// entries, the last one is T), then for every unit the first and the last
// wave that hold pages of it.
struct StreamTables {
  int32_t *range_tab, *unit_first, *unit_last;
  __host__ __device__ StreamTables(int32_t *page_prefix, int n_units) {
    range_tab = page_prefix + n_units + 1;
    unit_first = range_tab + STREAM_MAX_WG * 4 + 1;
    unit_last = unit_first + n_units;
  }
};

template <int D, int NP, bool NT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1)))
void decode_stream_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_new,
    const uint16_t *__restrict__ v_new, uint4 *kc, uint4 *vc, const int64_t *__restrict__ offsets,
    const int32_t *__restrict__ lens, int32_t *__restrict__ eff_len, int32_t *__restrict__ page_prefix,
    int *__restrict__ d_err, float *__restrict__ pm, float *__restrict__ pl, float *__restrict__ po,
    int n_units, int Hq, int Hkv, int G, float scale_log2, int skew) {
  constexpr int KK = D / 32, MB = D / 16, PSTRIDE = PAGE * (D / 8);  // uint4 per page
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 4, c = l & 15;
  const int hg = blockIdx.y;
  const bool want_app = k_new != nullptr;

  // ---- prologue: one trip to memory for lens / offsets, then everything the
  // waves need about the units (first page, token offset, length) lives in LDS
  __shared__ int s_pref[MAXU + 1];
  __shared__ int s_len[MAXU];        // length used by this step, bit 31 = a token is appended
  __shared__ int s_off[MAXU];        // offsets / CHUNK
  __shared__ int s_wtot[4];
  const bool publish = blockIdx.x == 0 && hg == 0;
  int64_t T;
  int lane_pref = 0x7fffffff;   // with at most 64 units: the first page of the lane's unit
  if (n_units <= 64) {
    // Few units: every wave builds the whole table by itself, a lane per unit,
    // so that no wave waits for another (the four waves write the same values
    // to the same words of LDS; a wave reads back what it wrote itself or the
    // identical word of a neighbour).
    int len = 0, pages = 0;
    if (l < n_units) {
      const int len_old = lens[l];
      const int64_t o0 = offsets[l], o1 = offsets[l + 1];
      const bool can = want_app && len_old < (int)(o1 - o0);
      len = len_old + (can ? 1 : 0);
      pages = (len + PAGE - 1) / PAGE;
      s_len[l] = len | (can ? (int)0x80000000 : 0);
      s_off[l] = (int)(o0 / CHUNK);
      if (publish && w == 0) {
        eff_len[l] = len;
        if (want_app && !can) atomicOr(d_err, 1);
      }
    }
    int incl = pages;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off);
      if (l >= off) incl += t;
    }
    const int total = __shfl(incl, 63);
    if (l < n_units) {
      lane_pref = incl - pages;
      s_pref[l] = lane_pref;
      if (publish && w == 0) page_prefix[l] = lane_pref;
    }
    if (l == 0) {
      s_pref[n_units] = total;
      if (publish && w == 0) page_prefix[n_units] = total;
    }
    T = total;
    // the wave's LDS writes above are read below, in program order
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  } else {
  const int upt = (n_units + 255) / 256;
  const int first = tid * upt;
  int sum = 0;
  for (int i = 0; i < upt; ++i) {
    const int u = first + i;
    if (u < n_units) {
      const int len_old = lens[u];
      const int64_t o0 = offsets[u], o1 = offsets[u + 1];
      const bool can = want_app && len_old < (int)(o1 - o0);
      const int len = len_old + (can ? 1 : 0);
      s_len[u] = len | (can ? (int)0x80000000 : 0);
      s_off[u] = (int)(o0 / CHUNK);
      sum += (len + PAGE - 1) / PAGE;
      if (publish) {
        eff_len[u] = len;
        if (want_app && !can) atomicOr(d_err, 1);
      }
    }
  }
  int incl = sum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (l >= off) incl += t;
  }
  if (l == 63) s_wtot[w] = incl;
  __syncthreads();
  int run = incl - sum;
  for (int ww = 0; ww < w; ++ww) run += s_wtot[ww];
  for (int i = 0; i < upt; ++i) {
    const int u = first + i;
    if (u < n_units) {
      s_pref[u] = run;
      if (publish) page_prefix[u] = run;
      run += ((s_len[u] & 0x7fffffff) + PAGE - 1) / PAGE;
    }
  }
  if (tid == 255) {
    s_pref[n_units] = run;
    if (publish) page_prefix[n_units] = run;
  }
  __syncthreads();
  T = s_pref[n_units];
  }
  const int W = gridDim.x * 4;
  const int wid = blockIdx.x * 4 + w;
  const int p0 = (int)range_start(wid, T, W, skew), p1 = (int)range_start(wid + 1, T, W, skew);
  const StreamTables tabs(page_prefix, n_units);
  const bool scribe = hg == 0 && l == 0;   // one lane per wave keeps the tables
  if (scribe) {
    tabs.range_tab[wid] = p0;
    if (wid == W - 1) tabs.range_tab[W] = p1;
  }
  if (p0 >= p1) return;

  // first unit of my range: largest u with s_pref[u] <= p0
  int u0;
  if (n_units <= 64) {
    // the lanes hold the prefixes: one vote instead of a chain of LDS reads
    u0 = __popcll(__ballot(lane_pref <= p0)) - 1;
  } else {
    int lo = 0, hi = n_units - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (s_pref[mid] <= p0) lo = mid; else hi = mid - 1;
    }
    u0 = lo;
  }

  // ---- fused append: the wave that owns the page receiving a unit's new token
  // stores it before requesting any page (it is the only reader of that page).
  if (want_app) {
    uint16_t *kc16 = reinterpret_cast<uint16_t *>(kc), *vc16 = reinterpret_cast<uint16_t *>(vc);
    bool stored = false;
    for (int u = u0; u < n_units && s_pref[u] < p1; ++u) {
      const int sl = s_len[u];
      if (sl >= 0) continue;                     // nothing appended to this unit
      const int len_old = (sl & 0x7fffffff) - 1;
      const int ap = s_pref[u] + len_old / PAGE;
      if (ap < p0 || ap >= p1) continue;
      const int64_t page = (int64_t)s_off[u] * CHUNK + (len_old / PAGE) * PAGE;
      const int t32 = len_old % PAGE, sb = t32 >> 4, r = t32 & 15;
      const int ga = (t32 & 15) >> 2, ea = 4 * (t32 >> 4) + (t32 & 3);
      for (int e = l; e < D; e += 64) {
        kc16[((size_t)page + sb * 16) * D + (size_t)((e >> 3) * 16 + r) * 8 + (e & 7)] = k_new[(size_t)u * D + e];
        vc16[(size_t)page * D + (size_t)((e >> 4) * 64 + ga * 16 + (e & 15)) * 8 + ea] = v_new[(size_t)u * D + e];
      }
      stored = true;
    }
    if (stored) __threadfence_block();   // the token is in place before its page is requested
  }

  // ---- ring of NP pages in flight
  PageRegs<D> ring[NP];
  // unit of the next page to request; its first page, end page and token offset
  // stay in registers so that a request costs no memory access of its own
  int u_ld = u0, pref_ld = s_pref[u0], next_ld = s_pref[u0 + 1];
  int64_t off_ld = (int64_t)s_off[u0] * CHUNK;
  auto locate = [&](int gp) {   // token slot of global page gp (pages are requested in ascending order)
    while (gp >= next_ld) {
      ++u_ld;
      pref_ld = next_ld;
      next_ld = s_pref[u_ld + 1];
      off_ld = (int64_t)s_off[u_ld] * CHUNK;
    }
    return (size_t)off_ld + (size_t)(gp - pref_ld) * PAGE;
  };
  auto request = [&](int gp, PageRegs<D> &r) {
    const size_t tok = locate(gp);
    load_page<D, NT>(kc + tok * (D / 8), vc + tok * (D / 8), l, r);
  };
  int u_at = -1;           // unit being accumulated
  int n_valid = 0;         // its token count
  int pref_at = 0, pref_next = 0;
  Frag qv[KK];
  float m_run = -INFINITY, l_run = 0.f;
  floatx4 acc[MB];
  const int slot_h = hg * 16 + c;

  auto flush = [&]() {
    const float l_tot = sum_lanes_16_32(l_run);
    if (slot_h < G) {
      const size_t pi = ((size_t)wid + u_at) * G + slot_h;
      if (g == 0) { pm[pi] = m_run; pl[pi] = l_tot; }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        *reinterpret_cast<floatx4 *>(po + pi * D + 16 * mb + 4 * g) = acc[mb];
    }
    if (scribe && pref_next <= p1) tabs.unit_last[u_at] = wid;   // the unit ends inside my range
  };
  // Vector memory operations complete in order, and the compiler places one
  // static wait per use: a load that only some paths issue (the query rows of
  // a new unit) would make every later wait assume the worst case and drain
  // the ring on every page.  The rare path therefore ends with all of its own
  // memory traffic complete, so that joining it changes nothing for the
  // common path.
  auto enter_unit = [&](int gp) {
    int u = u_at < 0 ? u0 : u_at;
    while (gp >= s_pref[u + 1]) ++u;
    u_at = u;
    pref_at = s_pref[u];
    pref_next = s_pref[u + 1];
    n_valid = s_len[u] & 0x7fffffff;
    if (scribe && gp == pref_at) tabs.unit_first[u] = wid;        // the unit starts inside my range
    const int b = u / Hkv, h = u % Hkv;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qv[kk].u = make_uint4(0, 0, 0, 0);
    if (slot_h < G) {
      const uint16_t *qp = q + ((size_t)b * Hq + (size_t)h * G + slot_h) * D;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) qv[kk].u = *reinterpret_cast<const uint4 *>(qp + 32 * kk + 8 * g);
    }
    m_run = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = floatx4{0.f, 0.f, 0.f, 0.f};
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): stores of flush() and the query loads are done
  };
  // One page: scores, request of the K tiles NP pages ahead, softmax and
  // values, request of the V tiles.
  auto page_step = [&](PageRegs<D> &r, int gp, bool more) {
    if (u_at < 0 || gp >= pref_next) {
      if (u_at >= 0) flush();
      enter_unit(gp);
    }
    floatx4 sc[2];
    page_scores<D>(r, qv, sc);
    size_t tok_next = 0;
    if (more) {
      tok_next = locate(gp + NP);
      load_page_k<D, NT>(kc + tok_next * (D / 8), l, r);
    }
    page_values<D>(r, sc, (gp - pref_at) * PAGE, n_valid, g, scale_log2, m_run, l_run, acc);
    if (more) load_page_v<D, NT>(vc + tok_next * (D / 8), l, r);
  };

  int gp0 = p0;
  if (p1 - p0 >= 2 * NP) {
    // steady state: every page of the loop refills its ring slot, so the number
    // of loads in flight at each wait is the same on every path and the waits
    // leave the other NP - 1 pages in flight
#pragma unroll
    for (int s = 0; s < NP; ++s) request(p0 + s, ring[s]);
    enter_unit(p0);
    for (; gp0 + 2 * NP <= p1; gp0 += NP) {
#pragma unroll
      for (int s = 0; s < NP; ++s) page_step(ring[s], gp0 + s, true);
    }
  } else {
#pragma unroll
    for (int s = 0; s < NP; ++s)
      if (p0 + s < p1) request(p0 + s, ring[s]);
  }
  // the last pages of the range (fewer than 2 NP), refilling only while pages remain
  for (; gp0 < p1; gp0 += NP) {
#pragma unroll
    for (int s = 0; s < NP; ++s) {
      const int gp = gp0 + s;
      if (gp < p1) page_step(ring[s], gp, gp + NP < p1);
    }
  }
  flush();
}

// Merge the partials of one (batch, query head): slots wave + unit for the waves
// whose page ranges meet the unit.  One block of 1024 threads = NCL slot lanes x
// D/4 channel lanes; slot lane c owns slots c, c+NCL, ... and requests UN of
// them at once (the partials sit in L2; the kernel is latency bound), reduces
// them with its own running maximum, and the NCL lane results are merged first
// inside each wave (lane exchanges), then over the waves in wave order -- one
// trip to memory, fixed summation order, reproducible.
template <int D>
__global__ __launch_bounds__(1024) void combine_stream_kernel(
    const float *__restrict__ pm, const float *__restrict__ pl, const float *__restrict__ po,
    const int32_t *__restrict__ page_prefix, const int32_t *__restrict__ eff_len,
    int32_t *__restrict__ lens_out, float *__restrict__ out, int n_units, int Hq, int Hkv, int G, int W) {
  constexpr int DL = D / 4, NCL = 1024 / DL, UN = 4;
  const int bq = blockIdx.x, tid = threadIdx.x;
  const int b = bq / Hq, hq = bq % Hq, h = hq / G, slot = hq % G;
  const int u = b * Hkv + h;
  if (lens_out != nullptr && slot == 0 && tid == 0) lens_out[u] = eff_len[u];
  const int64_t T = page_prefix[n_units];
  const int pa = page_prefix[u], pb = page_prefix[u + 1];
  // requested together with the prefixes (one trip to memory); meaningless for a unit without pages
  const StreamTables tabs(const_cast<int32_t *>(page_prefix), n_units);
  const int wa = tabs.unit_first[u], wb = tabs.unit_last[u];
  if (pa >= pb) {
    if (tid < D) out[(size_t)bq * D + tid] = 0.f;
    return;
  }
  const int nparts = wb - wa + 1;
  const size_t slot0 = (size_t)wa + u;
  const int dl = tid % DL, cl = tid / DL;
  __shared__ float4 red_o[NCL][DL];
  __shared__ float red_m[NCL], red_l[NCL];
  // a wave between the first and last owner wrote a partial unless its page range is empty
  const bool dense = T >= 2 * (int64_t)W;   // then every wave owns at least one page (skips the table look-ups)
  auto has_pages = [&](int i) {
    if (i >= nparts) return false;
    if (dense) return true;
    return tabs.range_tab[wa + i] < tabs.range_tab[wa + i + 1];
  };
  float m_run = -INFINITY, l_run = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int i0 = cl; i0 < nparts; i0 += NCL * UN) {
    float4 o[UN];
    float pmv[UN], plv[UN];
#pragma unroll
    for (int r = 0; r < UN; ++r) {
      const int i = i0 + r * NCL;
      const bool ok = has_pages(i);
      const size_t pi = (slot0 + (ok ? i : 0)) * G + slot;
      pmv[r] = ok ? pm[pi] : -INFINITY;
      plv[r] = ok ? pl[pi] : 0.f;
      o[r] = ok ? *reinterpret_cast<const float4 *>(po + pi * D + 4 * dl) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float m_new = m_run;
#pragma unroll
    for (int r = 0; r < UN; ++r) m_new = fmaxf(m_new, pmv[r]);
    if (m_new > -INFINITY) {
      const float a = __builtin_amdgcn_exp2f(m_run - m_new);
      acc.x *= a; acc.y *= a; acc.z *= a; acc.w *= a;
      l_run *= a;
#pragma unroll
      for (int r = 0; r < UN; ++r) {
        const float wgt = __builtin_amdgcn_exp2f(pmv[r] - m_new);
        acc.x += o[r].x * wgt; acc.y += o[r].y * wgt; acc.z += o[r].z * wgt; acc.w += o[r].w * wgt;
        l_run += plv[r] * wgt;
      }
      m_run = m_new;
    }
  }
  // the slot lanes of a wave (64 / DL of them) merge through lane exchanges
  // first -- both partners form the same sum -- so that the serial part below
  // goes over the block's sixteen waves instead of over all slot lanes
#pragma unroll
  for (int off = DL; off < 64; off <<= 1) {
    const float m_o = __shfl_xor(m_run, off), l_o = __shfl_xor(l_run, off);
    float4 a_o;
    a_o.x = __shfl_xor(acc.x, off); a_o.y = __shfl_xor(acc.y, off);
    a_o.z = __shfl_xor(acc.z, off); a_o.w = __shfl_xor(acc.w, off);
    const float m_new = fmaxf(m_run, m_o);
    const float a = m_run > -INFINITY ? __builtin_amdgcn_exp2f(m_run - m_new) : 0.f;
    const float b = m_o > -INFINITY ? __builtin_amdgcn_exp2f(m_o - m_new) : 0.f;
    acc.x = acc.x * a + a_o.x * b; acc.y = acc.y * a + a_o.y * b;
    acc.z = acc.z * a + a_o.z * b; acc.w = acc.w * a + a_o.w * b;
    l_run = l_run * a + l_o * b;
    m_run = m_new;
  }
  constexpr int NWV = 16;   // waves per block
  const int wv = tid >> 6;
  if ((tid & 63) < DL) {
    red_o[wv][dl] = acc;
    if (dl == 0) { red_m[wv] = m_run; red_l[wv] = l_run; }
  }
  __syncthreads();
  if (tid < DL) {
    float M = red_m[0];
#pragma unroll
    for (int cc = 1; cc < NWV; ++cc) M = fmaxf(M, red_m[cc]);
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = 0.f;
#pragma unroll
    for (int cc = 0; cc < NWV; ++cc) {
      const float wgt = __builtin_amdgcn_exp2f(red_m[cc] - M);   // 0 for lanes that saw no slot
      const float4 x = red_o[cc][tid];
      o.x += x.x * wgt; o.y += x.y * wgt; o.z += x.z * wgt; o.w += x.w * wgt;
      L += red_l[cc] * wgt;
    }
    const float inv = 1.f / L;
    *reinterpret_cast<float4 *>(out + (size_t)bq * D + 4 * tid) = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
  }
}

// Ring depth.  A wave can have at most 63 vector memory instructions in flight
// (the hardware counter is 6 bits) and a page is 16 of them, so rings deeper
// than 3 pages cannot be kept full; 2 pages measured fastest for 128-wide
// heads, at one wave per SIMD (fitting two waves into the register file costs
// spills and measured 5 % slower; 3 pages: 1 % slower).  Pages of 64-wide heads are
// half the size (8 instructions): 3 of them measured 3 % faster than 2 or 4.
template <int D>
constexpr int stream_ring_pages() { return D == 64 ? 3 : 2; }
// Fewest pages worth giving a wave: below this the launch is latency bound and
// extra waves only add partials for the combine kernel to read (measured on
// steps of 10-70 MB: 3 is 1-3 % faster than 4; with 2 the kernel itself gains
// another 1.5 us but the combine kernel loses more).
constexpr int STREAM_MIN_PAGES = 3;

template <int D, bool NT>
static void run_stream(taskkv_ctx *ctx, const Dims &dm, const uint16_t *q, const uint16_t *kn,
                       const uint16_t *vn, uint4 *kc, uint4 *vc, const int64_t *offsets, int32_t *lens,
                       int32_t *eff_len, int32_t *page_prefix, float *pm, float *pl, float *po,
                       float *out, int n_wg, bool fused, hipStream_t s) {
  const int skew = (n_wg & 1) ? 0 : ctx->stream_skew;
  const dim3 grid(n_wg, (dm.G + 15) / 16), block(256);
  const float scale_log2 = (float)(dm.scale * 1.4426950408889634);
  launch_attention(ctx, decode_stream_kernel<D, stream_ring_pages<D>(), NT>, grid, block,
                   s, q, kn, vn, kc, vc, offsets, lens, eff_len, page_prefix, ctx->d_err, pm, pl, po, dm.units,
                   dm.Hq, dm.Hkv, dm.G, scale_log2, skew);
  combine_stream_kernel<D><<<dim3(dm.B * dm.Hq), dim3(1024), 0, s>>>(
      pm, pl, po, page_prefix, eff_len, fused ? lens : nullptr, out, dm.units, dm.Hq, dm.Hkv, dm.G, n_wg * 4);
}

int launch_decode_stream(taskkv_ctx *ctx, const Dims &dm, const void *q, const void *k_new,
                         const void *v_new, void *k_cache, void *v_cache, int64_t capacity,
                         const int64_t *offsets, int32_t *lens, int32_t *eff_len, int32_t *page_prefix,
                         float *pm, float *pl, float *po, float *out, hipStream_t s) {
  const bool nt = (size_t)capacity * dm.D * 4 > NT_THRESHOLD_BYTES;
  const int variant = (dm.D == 64 ? 0 : 2) + (nt ? 1 : 0);
  if (!ctx->stream_wg[variant]) {
    // as many blocks as fit on the device at once, so that every wave is resident
    int per_cu = 0;
    hipError_t e;
    if (dm.D == 64)
      e = nt ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_stream_kernel<64, stream_ring_pages<64>(), true>, 256, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_stream_kernel<64, stream_ring_pages<64>(), false>, 256, 0);
    else
      e = nt ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_stream_kernel<128, stream_ring_pages<128>(), true>, 256, 0)
             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_stream_kernel<128, stream_ring_pages<128>(), false>, 256, 0);
    if (e != hipSuccess || per_cu < 1) return TASKKV_EHIP;
    int n = ctx->n_cu * per_cu;
    ctx->stream_wg[variant] = n > STREAM_MAX_WG ? STREAM_MAX_WG : n;
  }
  int n_wg = ctx->stream_wg[variant];
  {
    // capacity / PAGE bounds the pages of a step from above
    const int64_t want = (capacity / PAGE + 4 * STREAM_MIN_PAGES - 1) / (4 * STREAM_MIN_PAGES);
    if (want < n_wg) n_wg = want < 1 ? 1 : (int)want;
  }
  // The append is fused when one head slice covers the query group; otherwise
  // it runs as its own kernel first.
  const bool fused = k_new != nullptr && dm.G <= 16;
  if (k_new && !fused) {
    int rc = launch_append(dm, TASKKV_BF16, k_new, v_new, k_cache, v_cache, offsets, lens, ctx->d_err, s);
    if (rc) return rc;
  }
  auto qq = static_cast<const uint16_t *>(q);
  auto kn = fused ? static_cast<const uint16_t *>(k_new) : nullptr;
  auto vn = fused ? static_cast<const uint16_t *>(v_new) : nullptr;
  auto kc = static_cast<uint4 *>(k_cache), vc = static_cast<uint4 *>(v_cache);
  if (dm.D == 64) {
    if (nt) run_stream<64, true>(ctx, dm, qq, kn, vn, kc, vc, offsets, lens, eff_len, page_prefix, pm, pl, po, out, n_wg, fused, s);
    else run_stream<64, false>(ctx, dm, qq, kn, vn, kc, vc, offsets, lens, eff_len, page_prefix, pm, pl, po, out, n_wg, fused, s);
  } else {
    if (nt) run_stream<128, true>(ctx, dm, qq, kn, vn, kc, vc, offsets, lens, eff_len, page_prefix, pm, pl, po, out, n_wg, fused, s);
    else run_stream<128, false>(ctx, dm, qq, kn, vn, kc, vc, offsets, lens, eff_len, page_prefix, pm, pl, po, out, n_wg, fused, s);
  }
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
