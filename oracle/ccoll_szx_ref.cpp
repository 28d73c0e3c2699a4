// ccoll_szx_ref -- CPU oracle for the C-Coll SZx hot path.  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-threaded implementation of what the product library
// computes: the chunked SZx-style error-bounded compressor for float32, its
// decompressor (whole stream or an aligned range) and the per-round
// decompress + sum + recompress step of the compressed ring reduce-scatter.
// It shares no code with the HIP path and nothing in the product may call it;
// only tests, the smoke check and the bench's cpu_baseline leg use it.
//
// What it follows:
//   * C-Coll paper, Sec. III-E.2 ("Customize SZx ..."): data are compressed in
//     chunks of 5120 points; the compressed size of every chunk (4 bytes each)
//     is kept together at the front of the output buffer as an index, and the
//     decompressor walks a chunk-start pointer derived from those sizes.
//   * Sec. III-A.2 (collective computation framework) and Eq. 2: per round a
//     rank decompresses what it received, adds its local chunk (MPI_SUM on
//     floats) and compresses the sum again.
//   * Sec. III-B: after the data-movement framework every point is within the
//     error bound of the original.
//   * Table II: SZx's best ratio 124.1 = 512 B / (4 B + 1 bit), i.e. blocks of
//     128 floats whose constant form is one float plus one state bit.
//   * The paper does not print SZx's internals.  The block rules used here
//     (constant rule on half the value range, median, required-bit budget,
//     leading-byte coding against the previous element, one state bit per
//     block) are this project's stream definition "CSX1"; each rule is stated
//     where it is implemented.
//
// Pins (tests/test_oracle_*.py): the error bound on every element, the
// constant rule, bit-exact RAW round trips, closed-form sizes for constant
// input, two hand-derived byte streams, an independent slow decoder, the
// P*eb bound on chained reduce steps, range == slice of full decode; the Max /
// Min reduce steps against elementwise maximum / minimum followed by compress,
// their decisions on signed zeros, infinities and NaNs, and their P*eb bound.
// Unpinned: exact bytes on realistic data (the paper prints none).
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr int kBlock = 128;        // elements per block
constexpr int kChunk = 5120;       // elements per chunk (paper, Sec. III-E.2)
constexpr int kBlocksPerChunk = kChunk / kBlock;  // 40
constexpr size_t kHeader = 32;
constexpr size_t kMaxChunkPayload = 8 + 4 * 40 + 2 * 40 + 40 + 40 * (32 + 512);  // 22048

enum { OK = 0, EINVAL_ = -1, ENOSPC_ = -2, ECORRUPT_ = -3 };
enum BlockType { T_CONST = 0, T_NONCONST = 1, T_RAW = 2 };

inline uint32_t bits_of(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float float_of(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

// Unbiased exponent with denormals and zero mapped to -126.
inline int ex_of(float f) {
  int e = (int)((bits_of(f) >> 23) & 0xffu);
  if (e < 1) e = 1;
  return e - 127;
}

// Key that orders all finite floats (and +-0, -0 < +0) as unsigned integers.
inline uint32_t order_key(uint32_t b) { return (b & 0x80000000u) ? ~b : (b | 0x80000000u); }

// The error-bound contract is defined in this arithmetic.
inline bool dchk(float a, float b, float eb) {
  return std::fabs((double)a - (double)b) <= (double)eb;
}

inline bool eb_valid(float eb) { return std::isfinite(eb) && eb > 0.0f; }

// floor(log2(eb)) exactly, also for denormal eb.
inline int eb_exponent(float eb) { return std::ilogb(eb); }

struct BlockClass {
  int type;      // BlockType
  float mu;      // constant / median / +0
  int m;         // mantissa bits kept (NONCONST)
  int reqlen;    // 9+m, or 32 for RAW, 0 for CONST
};

BlockClass classify(const float* x, int len, float eb, int e_eb) {
  BlockClass r{T_RAW, 0.0f, 0, 32};
  // Any NaN / Inf makes the block RAW.
  for (int i = 0; i < len; ++i)
    if (((bits_of(x[i]) >> 23) & 0xffu) == 0xffu) return r;
  // min / max under the total order.
  float mn = x[0], mx = x[0];
  uint32_t kmn = order_key(bits_of(mn)), kmx = kmn;
  for (int i = 1; i < len; ++i) {
    uint32_t k = order_key(bits_of(x[i]));
    if (k < kmn) { kmn = k; mn = x[i]; }
    if (k > kmx) { kmx = k; mx = x[i]; }
  }
  volatile float d = mx - mn;  // volatile: keep each step a single fp32 rounding
  if (!std::isfinite(d)) return r;
  volatile float rad = 0.5f * d;
  volatile float muv = mn + rad;
  float mu = muv;
  // Constant rule: half the range within the bound, and the bound really
  // holds (in double) at both extremes.
  if (rad <= eb && dchk(mx, mu, eb) && dchk(mn, mu, eb)) {
    r.type = T_CONST; r.mu = mu; r.m = 0; r.reqlen = 0;
    return r;
  }
  volatile float va = mx - mu, vb = mn - mu;
  float vmax = std::fmax(std::fabs(va), std::fabs(vb));
  int e_v = ex_of(vmax);
  int e_M = ex_of(std::fmax(std::fabs(mn), std::fabs(mx)));
  int m = e_v - e_eb;
  if (m < 0) m = 0;
  if (m > 23) m = 23;
  // RAW when the bound lies below 4 ulp of the largest magnitude, when 16 or more mantissa bits would be
  // kept (4 bytes per element anyway), or when a value lies in the top binade: there the rounded centred
  // value plus the median can reach 2^128 and decode as Inf, which would break the bound of Sec. III-B
  // (e.g. {0, FLT_MAX} under a bound of 2^120).  Below the top binade |x| + abs_eb < 2^128 - 2^103.
  if (e_eb < e_M - 21 || m >= 16 || e_M >= 127) return r;  // RAW
  r.type = T_NONCONST; r.mu = mu; r.m = m; r.reqlen = 9 + m;
  return r;
}

// Codes one non-constant block body (lead codes then mid bytes) into out;
// returns the body size in bytes.
int encode_body(const float* x, int len, const BlockClass& bc, uint8_t* out) {
  const int reqlen = bc.reqlen;
  const int nbytes = (reqlen + 7) / 8;
  const int nlead = (len + 3) / 4;
  std::memset(out, 0, (size_t)nlead);
  uint8_t* mid = out + nlead;
  uint32_t prev = 0;
  for (int i = 0; i < len; ++i) {
    uint32_t t;
    if (bc.type == T_RAW) {
      t = bits_of(x[i]);
    } else {
      volatile float v = x[i] - bc.mu;
      uint32_t u = bits_of(v);
      const int m = bc.m;
      if (m < 23) {
        u = u + (1u << (22 - m));
        u &= ~((1u << (23 - m)) - 1u);
      }
      t = u >> (32 - reqlen);
    }
    // number of equal leading bytes in the nbytes-byte big-endian view
    int eq = 0;
    for (int b = 0; b < nbytes; ++b) {
      int sh = 8 * (nbytes - 1 - b);
      if (((t >> sh) & 0xffu) == ((prev >> sh) & 0xffu)) ++eq; else break;
    }
    int L = eq < 3 ? eq : 3;
    out[i >> 2] |= (uint8_t)(L << (2 * (i & 3)));
    for (int b = L; b < nbytes; ++b) *mid++ = (uint8_t)(t >> (8 * (nbytes - 1 - b)));
    prev = t;
  }
  return (int)(mid - out);
}

inline void put_u16(uint8_t* p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
inline void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
inline void put_u64(uint8_t* p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
inline uint16_t get_u16(const uint8_t* p) { return (uint16_t)(p[0] | (p[1] << 8)); }
inline uint32_t get_u32(const uint8_t* p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
inline uint64_t get_u64(const uint8_t* p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

inline size_t pad4(size_t v) { return (v + 3) & ~(size_t)3; }

// One chunk -> payload bytes in buf (capacity kMaxChunkPayload); returns size.
size_t encode_chunk(const float* x, int len, float eb, int e_eb, uint8_t* buf, int counts[3]) {
  const int nbc = (len + kBlock - 1) / kBlock;
  BlockClass cls[kBlocksPerChunk];
  uint64_t bitmap = 0;
  int k = 0;
  for (int j = 0; j < nbc; ++j) {
    int bl = len - j * kBlock; if (bl > kBlock) bl = kBlock;
    cls[j] = classify(x + j * kBlock, bl, eb, e_eb);
    if (counts) counts[cls[j].type]++;
    if (cls[j].type != T_CONST) { bitmap |= (uint64_t)1 << j; ++k; }
  }
  uint8_t* p = buf;
  put_u64(p, bitmap); p += 8;
  for (int j = 0; j < nbc; ++j) { put_u32(p, bits_of(cls[j].mu)); p += 4; }
  uint8_t* p_bsize = p;
  uint8_t* p_req = p + 2 * k;
  size_t meta = pad4((size_t)(8 + 4 * nbc + 3 * k));
  std::memset(p, 0, meta - (size_t)(8 + 4 * nbc));
  uint8_t* body = buf + meta;
  int idx = 0;
  for (int j = 0; j < nbc; ++j) {
    if (cls[j].type == T_CONST) continue;
    int bl = len - j * kBlock; if (bl > kBlock) bl = kBlock;
    int bs = encode_body(x + j * kBlock, bl, cls[j], body);
    put_u16(p_bsize + 2 * idx, (uint16_t)bs);
    p_req[idx] = (uint8_t)cls[j].reqlen;
    body += bs;
    ++idx;
  }
  size_t used = (size_t)(body - buf);
  size_t total = pad4(used);
  std::memset(buf + used, 0, total - used);
  return total;
}

struct Header {
  uint64_t n, total;
  uint32_t nchunks, eb_bits;
};

// Validates header + index; on success fills h and the exclusive prefix of
// chunk sizes (offsets from the start of the payload area).
int parse_header(const uint8_t* in, size_t in_bytes, Header& h, std::vector<uint64_t>* offs) {
  if (in_bytes < kHeader) return ECORRUPT_;
  if (!(in[0] == 'C' && in[1] == 'S' && in[2] == 'X' && in[3] == '1')) return ECORRUPT_;
  if (get_u16(in + 4) != kBlock || get_u16(in + 6) != kChunk) return ECORRUPT_;
  h.n = get_u64(in + 8);
  h.eb_bits = get_u32(in + 16);
  h.nchunks = get_u32(in + 20);
  h.total = get_u64(in + 24);
  if (h.n > ((uint64_t)1 << 31)) return ECORRUPT_;
  if (!eb_valid(float_of(h.eb_bits))) return ECORRUPT_;
  if ((uint64_t)h.nchunks != (h.n + kChunk - 1) / kChunk) return ECORRUPT_;
  uint64_t front = kHeader + 4ull * h.nchunks;
  if (h.total < front || h.total > in_bytes) return ECORRUPT_;
  uint64_t sum = 0;
  if (offs) offs->resize((size_t)h.nchunks + 1);
  for (uint32_t c = 0; c < h.nchunks; ++c) {
    uint32_t sz = get_u32(in + kHeader + 4ull * c);
    uint64_t len = h.n - (uint64_t)c * kChunk; if (len > kChunk) len = kChunk;
    uint64_t nbc = (len + kBlock - 1) / kBlock;
    if ((sz & 3u) || sz < 8 + 4 * nbc || sz > kMaxChunkPayload) return ECORRUPT_;
    if (offs) (*offs)[c] = sum;
    sum += sz;
  }
  if (offs) (*offs)[h.nchunks] = sum;
  if (sum != h.total - front) return ECORRUPT_;
  return OK;
}

// Decodes blocks [b0, b1) of one chunk (len elements, payload p of size sz)
// into out (element 0 of out = first element of block b0).
int decode_chunk(const uint8_t* p, size_t sz, int len, int b0, int b1, float* out) {
  const int nbc = (len + kBlock - 1) / kBlock;
  if (sz < (size_t)(8 + 4 * nbc)) return ECORRUPT_;
  uint64_t bitmap = get_u64(p);
  if (nbc < 64 && (bitmap >> nbc) != 0) return ECORRUPT_;
  int k = 0;
  for (int j = 0; j < nbc; ++j) k += (int)((bitmap >> j) & 1u);
  size_t meta = pad4((size_t)(8 + 4 * nbc + 3 * k));
  if (meta > sz) return ECORRUPT_;
  const uint8_t* p_mu = p + 8;
  const uint8_t* p_bsize = p_mu + 4 * nbc;
  const uint8_t* p_req = p_bsize + 2 * k;
  size_t bodies = 0;
  for (int i = 0; i < k; ++i) {
    int rq = p_req[i];
    if (!((rq >= 9 && rq <= 24) || rq == 32)) return ECORRUPT_;
    bodies += get_u16(p_bsize + 2 * i);
  }
  if (pad4(meta + bodies) != sz) return ECORRUPT_;
  size_t off = meta;
  int idx = 0;
  for (int j = 0; j < nbc; ++j) {
    int bl = len - j * kBlock; if (bl > kBlock) bl = kBlock;
    bool nonconst = (bitmap >> j) & 1u;
    float mu = float_of(get_u32(p_mu + 4 * j));
    if (!nonconst) {
      if (j >= b0 && j < b1) for (int i = 0; i < bl; ++i) out[(j - b0) * kBlock + i] = mu;
      continue;
    }
    int bs = get_u16(p_bsize + 2 * idx);
    int reqlen = p_req[idx];
    ++idx;
    if (j >= b0 && j < b1) {
      const int nbytes = (reqlen + 7) / 8;
      const int nlead = (bl + 3) / 4;
      if (bs < nlead) return ECORRUPT_;
      const uint8_t* lead = p + off;
      const uint8_t* mid = lead + nlead;
      const uint8_t* end = p + off + bs;
      uint32_t prev = 0;
      for (int i = 0; i < bl; ++i) {
        int L = (lead[i >> 2] >> (2 * (i & 3))) & 3;
        if (L > nbytes) return ECORRUPT_;
        if (mid + (nbytes - L) > end) return ECORRUPT_;
        uint32_t t = 0;
        for (int b = 0; b < nbytes; ++b) {
          int sh = 8 * (nbytes - 1 - b);
          uint32_t byte = (b < L) ? ((prev >> sh) & 0xffu) : (uint32_t)(*mid++);
          t |= byte << sh;
        }
        prev = t;
        float v;
        if (reqlen == 32) {
          v = float_of(t);
        } else {
          volatile float s = float_of(t << (32 - reqlen)) + mu;
          v = s;
        }
        out[(j - b0) * kBlock + i] = v;
      }
      if (mid != end) return ECORRUPT_;
    }
    off += (size_t)bs;
  }
  return OK;
}

}  // namespace

extern "C" {

size_t ccoll_ref_max_compressed_bytes(size_t n) {
  size_t nchunks = (n + kChunk - 1) / kChunk;
  return kHeader + nchunks * (kMaxChunkPayload + 4);
}

// counts (optional, 3 ints): number of CONST / NONCONST / RAW blocks.
int ccoll_ref_compress_stats(const float* in, size_t n, float abs_eb, void* out_, size_t cap,
                             size_t* out_bytes, long long* counts) {
  if (!out_ || !out_bytes || (!in && n) || !eb_valid(abs_eb) || n > ((size_t)1 << 31)) return EINVAL_;
  uint8_t* out = (uint8_t*)out_;
  const int e_eb = eb_exponent(abs_eb);
  const size_t nchunks = (n + kChunk - 1) / kChunk;
  const size_t front = kHeader + 4 * nchunks;
  if (cap < front) return ENOSPC_;
  std::vector<uint8_t> buf(kMaxChunkPayload);
  size_t pos = front;
  int cnt[3] = {0, 0, 0};
  long long tot[3] = {0, 0, 0};
  for (size_t c = 0; c < nchunks; ++c) {
    size_t len = n - c * kChunk; if (len > kChunk) len = kChunk;
    cnt[0] = cnt[1] = cnt[2] = 0;
    size_t sz = encode_chunk(in + c * kChunk, (int)len, abs_eb, e_eb, buf.data(), cnt);
    for (int i = 0; i < 3; ++i) tot[i] += cnt[i];
    if (pos + sz > cap) return ENOSPC_;
    std::memcpy(out + pos, buf.data(), sz);
    put_u32(out + kHeader + 4 * c, (uint32_t)sz);
    pos += sz;
  }
  out[0] = 'C'; out[1] = 'S'; out[2] = 'X'; out[3] = '1';
  put_u16(out + 4, kBlock);
  put_u16(out + 6, kChunk);
  put_u64(out + 8, (uint64_t)n);
  put_u32(out + 16, bits_of(abs_eb));
  put_u32(out + 20, (uint32_t)nchunks);
  put_u64(out + 24, (uint64_t)pos);
  *out_bytes = pos;
  if (counts) for (int i = 0; i < 3; ++i) counts[i] = tot[i];
  return OK;
}

int ccoll_ref_compress(const float* in, size_t n, float abs_eb, void* out, size_t cap, size_t* out_bytes) {
  return ccoll_ref_compress_stats(in, n, abs_eb, out, cap, out_bytes, nullptr);
}

int ccoll_ref_decompress_range(const void* in_, size_t in_bytes, size_t first, size_t count, float* out) {
  if (!in_ || (!out && count)) return EINVAL_;
  if (first % kBlock) return EINVAL_;
  const uint8_t* in = (const uint8_t*)in_;
  Header h;
  std::vector<uint64_t> offs;
  int rc = parse_header(in, in_bytes, h, &offs);
  if (rc) return rc;
  if (first > h.n || count > h.n - first) return EINVAL_;
  if (count == 0) return OK;
  const size_t front = kHeader + 4ull * h.nchunks;
  const size_t last = first + count;  // exclusive
  std::vector<float> tmp(kChunk);
  for (size_t c = first / kChunk; c * kChunk < last; ++c) {
    size_t cbeg = c * kChunk;
    size_t len = h.n - cbeg; if (len > kChunk) len = kChunk;
    size_t lo = first > cbeg ? first - cbeg : 0;           // multiple of 128
    size_t hi = last < cbeg + len ? last - cbeg : len;      // exclusive, element
    int b0 = (int)(lo / kBlock);
    int b1 = (int)((hi + kBlock - 1) / kBlock);
    uint32_t sz = get_u32(in + kHeader + 4 * c);
    rc = decode_chunk(in + front + offs[c], sz, (int)len, b0, b1, tmp.data());
    if (rc) return rc;
    std::memcpy(out + (cbeg + lo - first), tmp.data(), (hi - lo) * sizeof(float));
  }
  return OK;
}

int ccoll_ref_decompress(const void* in, size_t in_bytes, float* out, size_t n) {
  if (!in || (!out && n)) return EINVAL_;
  Header h;
  int rc = parse_header((const uint8_t*)in, in_bytes, h, nullptr);
  if (rc) return rc;
  if (h.n != n) return ECORRUPT_;
  return ccoll_ref_decompress_range(in, in_bytes, 0, n, out);
}

// One round of the compressed ring reduce-scatter with the reduction op of the collective (Sec. III-B names
// Sum, Average, Max and Min; Average is a Sum divided once at the end by the caller):
//   op 0: s = local + x'  -- one fp32 round-to-nearest add (Eq. 2)
//   op 1: s = max(local, x'),  op 2: s = min(local, x')  under the total order of the bit patterns that the
//         block classification uses (-NaN < -Inf < ... < -0 < +0 < ... < +Inf < +NaN), so that the result does
//         not depend on the order of the operands and NaN / signed zeros are decided, not left to the compiler.
int ccoll_ref_reduce_step_op(int op, const float* local, size_t n, const void* cin, size_t cin_bytes, float abs_eb,
                             void* cout, size_t cap, size_t* out_bytes) {
  if ((!local && n) || !cin || !cout || !out_bytes || !eb_valid(abs_eb) || op < 0 || op > 2) return EINVAL_;
  std::vector<float> s(n ? n : 1);
  int rc = ccoll_ref_decompress(cin, cin_bytes, s.data(), n);
  if (rc) return rc;
  for (size_t i = 0; i < n; ++i) {
    if (op == 0) {
      volatile float t = local[i] + s[i];
      s[i] = t;
    } else {
      uint32_t a, b;
      std::memcpy(&a, &local[i], 4); std::memcpy(&b, &s[i], 4);
      const bool a_greater = order_key(a) > order_key(b);
      const uint32_t r = (op == 1) == a_greater ? a : b;
      std::memcpy(&s[i], &r, 4);
    }
  }
  return ccoll_ref_compress(s.data(), n, abs_eb, cout, cap, out_bytes);
}

int ccoll_ref_reduce_step(const float* local, size_t n, const void* cin, size_t cin_bytes, float abs_eb,
                          void* cout, size_t cap, size_t* out_bytes) {
  return ccoll_ref_reduce_step_op(0, local, n, cin, cin_bytes, abs_eb, cout, cap, out_bytes);
}

// Classification of one block, exposed so tests can pin the constant rule.
// type: 0 CONST, 1 NONCONST, 2 RAW.
int ccoll_ref_classify_block(const float* x, int len, float abs_eb, int* type, float* mu, int* reqlen) {
  if (!x || len < 1 || len > kBlock || !eb_valid(abs_eb)) return EINVAL_;
  BlockClass bc = classify(x, len, abs_eb, eb_exponent(abs_eb));
  *type = bc.type; *mu = bc.mu; *reqlen = bc.reqlen;
  return OK;
}

}  // extern "C"
