// Entropy stage of the delta (Sec. 6, "Encoding Delta"), host code outside the timed path: every
// group of the regrouped delta stream is run-length encoded -- a run of r equal values v becomes the
// token -v, followed by the token +r when r > 1 -- and the tokens are Huffman coded, one code per
// group (the groups are encoded separately).
//
// Container (little-endian):
//   header   u32 magic "IDE1", u32 n_groups, u64 n, u32 delta_bits, u32 0
//   group    u64 n_values, u64 n_tokens, u64 payload_bits, u32 n_sym, u32 0,
//            n_sym x { i32 token, u32 code length }   in canonical order (length, then token),
//            ceil(payload_bits / 8) bytes: the codes, most significant code bit first, filling
//            every byte from bit 0 upwards
// A group with one distinct token has code length 0 and no payload: n_tokens fixes the sequence.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "../../include/inshr.h"

namespace {

struct ValueReader { // delta values of a stream: packed w-bit fields or one u16 per value
    const uint64_t *packed;
    const uint16_t *plain;
    uint32_t w;
    uint32_t get(uint64_t i) const
    {
        if (plain) return plain[i];
        const uint64_t bit = i * w, wd = bit >> 6;
        const uint32_t sh = (uint32_t)(bit & 63u);
        uint64_t x = packed[wd] >> sh;
        if (sh + w > 64u) x |= packed[wd + 1] << (64u - sh);
        return (uint32_t)(x & ((1ull << w) - 1ull));
    }
};

struct Sym {
    int32_t token;
    uint32_t len;
    uint64_t count;
    uint64_t code;
};

// run-length tokens of values [lo, hi)
void rle(const ValueReader &rd, uint64_t lo, uint64_t hi, std::vector<int32_t> &tok)
{
    tok.clear();
    uint64_t i = lo;
    while (i < hi) {
        const uint32_t v = rd.get(i);
        uint64_t j = i + 1;
        while (j < hi && rd.get(j) == v) j++;
        uint64_t r = j - i;
        while (r) { // a run longer than a token can hold is cut
            const uint64_t part = r > 0x7fffffffull ? 0x7fffffffull : r;
            tok.push_back(-(int32_t)v);
            if (part > 1) tok.push_back((int32_t)part);
            r -= part;
        }
        i = j;
    }
}

// Huffman code lengths by the two-queue construction on the symbols in ascending (count, token)
// order (leaves before merged nodes on equal weight), then canonical codes in (length, token) order
void build_code(const std::vector<int32_t> &tok, std::vector<Sym> &syms)
{
    syms.clear();
    std::unordered_map<int32_t, uint64_t> freq;
    freq.reserve(1024);
    for (int32_t t : tok) freq[t]++;
    syms.reserve(freq.size());
    for (auto &kv : freq) syms.push_back(Sym{kv.first, 0u, kv.second, 0ull});
    const size_t k = syms.size();
    if (k <= 1) return;
    std::sort(syms.begin(), syms.end(), [](const Sym &a, const Sym &b) {
        return a.count != b.count ? a.count < b.count : a.token < b.token;
    });
    // nodes 0..k-1 are the leaves, k.. the merged ones in creation order (weights ascending)
    std::vector<uint64_t> weight(2 * k - 1);
    std::vector<uint32_t> parent(2 * k - 1, 0u);
    for (size_t i = 0; i < k; i++) weight[i] = syms[i].count;
    size_t leaf = 0, node = k, made = k;
    auto take = [&]() -> size_t {
        if (leaf < k && (node >= made || weight[leaf] <= weight[node])) return leaf++;
        return node++;
    };
    while (made < 2 * k - 1) {
        const size_t a = take(), b = take();
        weight[made] = weight[a] + weight[b];
        parent[a] = parent[b] = (uint32_t)made;
        made++;
    }
    std::vector<uint32_t> depth(2 * k - 1, 0u);
    for (size_t i = 2 * k - 2; i-- > 0;) depth[i] = depth[parent[i]] + 1u;
    for (size_t i = 0; i < k; i++) syms[i].len = depth[i];
    std::sort(syms.begin(), syms.end(), [](const Sym &a, const Sym &b) {
        return a.len != b.len ? a.len < b.len : a.token < b.token;
    });
    uint64_t code = 0;
    uint32_t len = syms[0].len;
    for (size_t i = 0; i < k; i++) {
        code <<= (syms[i].len - len);
        len = syms[i].len;
        syms[i].code = code++;
    }
}

struct BitWriter {
    uint8_t *p;
    uint64_t bit = 0;
    void put(uint64_t code, uint32_t len)
    {
        for (uint32_t b = len; b-- > 0;) {
            if ((code >> b) & 1ull) p[bit >> 3] |= (uint8_t)(1u << (bit & 7u));
            bit++;
        }
    }
};

template <class T> void put(uint8_t *&p, T v)
{
    memcpy(p, &v, sizeof(T));
    p += sizeof(T);
}
template <class T> bool get(const uint8_t *&p, const uint8_t *end, T &v)
{
    if ((size_t)(end - p) < sizeof(T)) return false;
    memcpy(&v, p, sizeof(T));
    p += sizeof(T);
    return true;
}

constexpr uint32_t MAGIC = 0x31454449u; // "IDE1"

int encode(const ValueReader &rd, uint64_t n, uint32_t delta_bits, const uint64_t *group_off,
           uint32_t n_groups, uint8_t *out, uint64_t out_cap, uint64_t *out_bytes,
           inshr_entropy_stats *stats)
{
    if (!group_off || !out_bytes || n_groups == 0 || delta_bits < 1 || delta_bits > 16) return INSHR_E_ARG;
    if (group_off[0] != 0 || group_off[n_groups] != n) return INSHR_E_SHAPE;
    for (uint32_t g = 0; g < n_groups; g++)
        if (group_off[g] > group_off[g + 1]) return INSHR_E_SHAPE;
    inshr_entropy_stats st;
    memset(&st, 0, sizeof(st));
    uint8_t *p = out;
    uint64_t used = 24;
    if (out && out_cap >= used) {
        put<uint32_t>(p, MAGIC);
        put<uint32_t>(p, n_groups);
        put<uint64_t>(p, n);
        put<uint32_t>(p, delta_bits);
        put<uint32_t>(p, 0u);
    }
    std::vector<int32_t> tok;
    std::vector<Sym> syms;
    std::unordered_map<int32_t, uint32_t> index;
    for (uint32_t g = 0; g < n_groups; g++) {
        rle(rd, group_off[g], group_off[g + 1], tok);
        build_code(tok, syms);
        uint64_t payload_bits = 0;
        for (const Sym &s : syms) payload_bits += s.count * s.len;
        const uint64_t need = 32 + 8ull * syms.size() + (payload_bits + 7) / 8;
        st.n_tokens += tok.size();
        st.table_bytes += 32 + 8ull * syms.size();
        st.payload_bytes += (payload_bits + 7) / 8;
        if (out && used + need <= out_cap) {
            put<uint64_t>(p, group_off[g + 1] - group_off[g]);
            put<uint64_t>(p, (uint64_t)tok.size());
            put<uint64_t>(p, payload_bits);
            put<uint32_t>(p, (uint32_t)syms.size());
            put<uint32_t>(p, 0u);
            index.clear();
            for (size_t i = 0; i < syms.size(); i++) {
                put<int32_t>(p, syms[i].token);
                put<uint32_t>(p, syms[i].len);
                index[syms[i].token] = (uint32_t)i;
            }
            const uint64_t nbytes = (payload_bits + 7) / 8;
            memset(p, 0, nbytes);
            if (payload_bits) {
                BitWriter bw{p};
                for (int32_t t : tok) {
                    const Sym &s = syms[index[t]];
                    bw.put(s.code, s.len);
                }
            }
            p += nbytes;
        }
        used += need;
    }
    *out_bytes = used;
    if (stats) *stats = st;
    return (out && used <= out_cap) ? INSHR_OK : INSHR_E_CAPACITY;
}

} // namespace

extern "C" {

int inshr_entropy_encode(const uint64_t *packed, const uint16_t *values, uint64_t n,
                         uint32_t delta_bits, const uint64_t *group_off, uint32_t n_groups,
                         uint8_t *out, uint64_t out_cap, uint64_t *out_bytes,
                         inshr_entropy_stats *stats)
{
    if ((packed == nullptr) == (values == nullptr)) return INSHR_E_ARG; // exactly one of the two
    ValueReader rd{packed, values, delta_bits};
    return encode(rd, n, delta_bits, group_off, n_groups, out, out_cap, out_bytes, stats);
}

int inshr_entropy_decode(const uint8_t *in, uint64_t in_bytes, uint64_t n, uint32_t delta_bits,
                         uint32_t n_groups, uint64_t *packed, uint16_t *values, uint64_t *group_off)
{
    if (!in || (packed == nullptr) == (values == nullptr)) return INSHR_E_ARG;
    const uint8_t *p = in, *end = in + in_bytes;
    uint32_t magic = 0, G = 0, w = 0, zero = 0;
    uint64_t nn = 0;
    if (!get(p, end, magic) || !get(p, end, G) || !get(p, end, nn) || !get(p, end, w) || !get(p, end, zero))
        return INSHR_E_SHAPE;
    if (magic != MAGIC || G != n_groups || nn != n || w != delta_bits || w < 1 || w > 16) return INSHR_E_SHAPE;
    if (packed) memset(packed, 0, ((n * w + 63) / 64) * 8);
    uint64_t pos = 0; // values written so far
    std::vector<Sym> syms;
    auto emit = [&](uint32_t v) {
        if (values) {
            values[pos] = (uint16_t)v;
        } else {
            const uint64_t bit = pos * w, wd = bit >> 6;
            const uint32_t sh = (uint32_t)(bit & 63u);
            packed[wd] |= (uint64_t)v << sh;
            if (sh + w > 64u) packed[wd + 1] |= (uint64_t)v >> (64u - sh);
        }
        pos++;
    };
    for (uint32_t g = 0; g < G; g++) {
        uint64_t n_values = 0, n_tokens = 0, payload_bits = 0;
        uint32_t n_sym = 0;
        if (!get(p, end, n_values) || !get(p, end, n_tokens) || !get(p, end, payload_bits) ||
            !get(p, end, n_sym) || !get(p, end, zero))
            return INSHR_E_SHAPE;
        if (group_off) group_off[g] = pos;
        if (pos + n_values > n || (uint64_t)(end - p) < 8ull * n_sym) return INSHR_E_SHAPE;
        syms.resize(n_sym);
        for (uint32_t i = 0; i < n_sym; i++) {
            get(p, end, syms[i].token);
            get(p, end, syms[i].len);
            if (syms[i].len > 63u || (i && syms[i].len < syms[i - 1].len)) return INSHR_E_SHAPE;
        }
        const uint64_t nbytes = (payload_bits + 7) / 8;
        if ((uint64_t)(end - p) < nbytes) return INSHR_E_SHAPE;
        // canonical decoding: first code and first symbol of every length
        uint64_t first_code[65], count[65];
        uint32_t first_sym[65];
        memset(count, 0, sizeof(count));
        for (uint32_t i = 0; i < n_sym; i++) count[syms[i].len]++;
        {
            uint64_t code = 0;
            uint32_t s = 0;
            for (uint32_t l = 0; l <= 64; l++) {
                first_code[l] = code;
                first_sym[l] = s;
                code = (code + count[l]) << 1;
                s += (uint32_t)count[l];
            }
        }
        const uint64_t start = pos;
        uint64_t bit = 0;
        uint32_t last = 0;
        bool have_last = false;
        for (uint64_t t = 0; t < n_tokens; t++) {
            int32_t token;
            if (n_sym == 1) {
                token = syms[0].token;
            } else {
                uint64_t code = 0;
                uint32_t l = 0;
                for (;;) {
                    if (bit >= payload_bits || l >= 63u) return INSHR_E_SHAPE;
                    code = (code << 1) | ((p[bit >> 3] >> (bit & 7u)) & 1u);
                    bit++;
                    l++;
                    if (count[l] && code >= first_code[l] && code - first_code[l] < count[l]) {
                        token = syms[first_sym[l] + (uint32_t)(code - first_code[l])].token;
                        break;
                    }
                }
            }
            if (token <= 0) {
                last = (uint32_t)(-token);
                have_last = true;
                if (last >> w || pos - start >= n_values) return INSHR_E_SHAPE;
                emit(last);
            } else {
                if (!have_last || pos - start + (uint64_t)(token - 1) > n_values) return INSHR_E_SHAPE;
                for (int32_t r = 1; r < token; r++) emit(last);
            }
        }
        if (pos - start != n_values) return INSHR_E_SHAPE;
        p += nbytes;
    }
    if (group_off) group_off[G] = pos;
    return pos == n ? INSHR_OK : INSHR_E_SHAPE;
}

} // extern "C"
