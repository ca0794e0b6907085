// Trace loading: JSON-lines parser, array import, candidate-independent preprocessing.
//
// The replay input is a Mooncake-style trace (Sec. 3 "Dataset": per-request timestamps, request metadata,
// block hash ids).  Everything that does not depend on the candidate weights is done here once: hash ids
// are renumbered densely (1 + order of first appearance), repeated ids inside one request are flagged, and
// the trace is classified as chain-consistent or not.
#include <cerrno>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <limits>
#include <new>
#include <string>

#include "internal.h"

namespace gorgo {

static thread_local std::string g_err;

int fail(int code, const std::string& msg) {
    g_err = msg;
    return code;
}
void clear_error() { g_err.clear(); }

namespace {

// Open-addressed int64 -> uint32 map (linear probing, grows by doubling); value 0 means empty.
class IdMap {
  public:
    IdMap() { resize(1 << 12); }
    // returns the dense key of id, assigning the next one on first sight
    uint32_t get_or_add(int64_t id, bool* added) {
        if ((count_ + 1) * 2 > cap_) resize(cap_ * 2);
        size_t h = mix((uint64_t)id) & (cap_ - 1);
        while (val_[h] != 0) {
            if (key_[h] == id) { *added = false; return val_[h]; }
            h = (h + 1) & (cap_ - 1);
        }
        key_[h] = id;
        val_[h] = (uint32_t)(++count_);
        *added = true;
        return val_[h];
    }
    size_t size() const { return count_; }

  private:
    static uint64_t mix(uint64_t x) {
        x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ULL;
        x ^= x >> 27; x *= 0x94d049bb133111ebULL;
        return x ^ (x >> 31);
    }
    void resize(size_t ncap) {
        std::vector<int64_t> ok;
        std::vector<uint32_t> ov;
        ok.swap(key_);
        ov.swap(val_);
        key_.assign(ncap, 0);
        val_.assign(ncap, 0);
        size_t ocap = cap_;
        cap_ = ncap;
        for (size_t i = 0; i < ocap; ++i) {
            if (!ov[i]) continue;
            size_t h = mix((uint64_t)ok[i]) & (cap_ - 1);
            while (val_[h] != 0) h = (h + 1) & (cap_ - 1);
            key_[h] = ok[i];
            val_[h] = ov[i];
        }
    }
    std::vector<int64_t> key_;
    std::vector<uint32_t> val_;
    size_t cap_ = 0, count_ = 0;
};

// Fills key/first/statistics from the raw ids.  Returns 0 or an error code.
int preprocess(gorgo_trace* t, const int64_t* hash_ids) {
    const int64_t N = t->N;
    const int64_t total = t->blk_off[N];
    t->total_blocks = total;
    t->key.resize((size_t)total);
    t->first.resize((size_t)total);
    IdMap map;
    // for chain consistency: the (predecessor key, position) each key was first seen with
    std::vector<uint32_t> parent;
    std::vector<uint32_t> pos;
    parent.push_back(0);
    pos.push_back(0);
    // per-request duplicate detection: last request index in which a key was seen
    std::vector<int64_t> seen_in;
    seen_in.push_back(-1);
    std::vector<uint32_t> nchild;    // distinct successors of a key
    std::vector<uint8_t> ends;       // some request ends at this key
    nchild.push_back(0);
    ends.push_back(0);
    bool consistent = true;
    int32_t max_blocks = 0, max_distinct = 0;
    for (int64_t r = 0; r < N; ++r) {
        const int64_t b = t->blk_off[r], e = t->blk_off[r + 1];
        const int64_t n = e - b;
        if (n > max_blocks) max_blocks = (int32_t)n;
        int32_t distinct = 0;
        uint32_t prev = 0;
        for (int64_t k = 0; k < n; ++k) {
            bool added = false;
            uint32_t key = map.get_or_add(hash_ids[b + k], &added);
            if (map.size() >= 0xFFFFFFF0ull) return fail(GORGO_ERR_INVALID_ARG, "too many distinct hash ids");
            if (added) {
                parent.push_back(prev);
                pos.push_back((uint32_t)k);
                seen_in.push_back(-1);
                nchild.push_back(0);
                ends.push_back(0);
                if (prev) ++nchild[prev];
            } else if (parent[key] != prev || pos[key] != (uint32_t)k) {
                consistent = false;
            }
            const bool dup = seen_in[key] == r;
            if (dup) consistent = false;
            else ++distinct;
            seen_in[key] = r;
            t->key[(size_t)(b + k)] = key;
            t->first[(size_t)(b + k)] = dup ? 0 : 1;
            prev = key;
        }
        if (prev) ends[prev] = 1;
        if (distinct > max_distinct) max_distinct = distinct;
    }
    t->max_blocks = max_blocks;
    t->max_distinct = max_distinct;
    t->unique_ids = (int64_t)map.size();
    t->chain_consistent = consistent;
    t->seg_off.clear();
    t->seg.clear();
    t->n_segments = 0;
    t->n_slots = 0;
    if (!consistent) return GORGO_OK;

    // Chain-consistent traces: the keys form a forest and every request is a root-to-node path.  Cut the
    // forest into segments -- maximal runs of keys with a single successor and no request ending inside --
    // so that every request is a whole number of segments and all blocks of a segment are always touched
    // together.  Keys are numbered in order of first appearance, so a predecessor precedes its successors.
    const size_t U = map.size();
    std::vector<int32_t> seg_of(U + 1, 0);
    int64_t nseg = 0;
    for (size_t k = 1; k <= U; ++k) {
        const uint32_t par = parent[k];
        if (par == 0 || nchild[par] > 1 || ends[par]) seg_of[k] = (int32_t)(nseg++);
        else seg_of[k] = seg_of[par];
        if (nseg >= 0x7FFFFFF0) return fail(GORGO_ERR_INVALID_ARG, "too many segments");
    }
    t->n_segments = nseg;
    t->seg_off.resize((size_t)N + 1);
    t->seg_off[0] = 0;
    for (int64_t r = 0; r < N; ++r) {
        const int64_t b = t->blk_off[r], e = t->blk_off[r + 1];
        for (int64_t k = b; k < e; ++k) {
            const int32_t sg = seg_of[t->key[(size_t)k]];
            if (k + 1 == e || seg_of[t->key[(size_t)k + 1]] != sg) t->seg.push_back(gorgo::SegRef{sg, (int32_t)(k + 1 - b)});
        }
        t->seg_off[(size_t)r + 1] = (int64_t)t->seg.size();
    }

    // Row slots.  The replay keeps one row of cells per segment, but a segment only matters between the first and
    // the last request that reference it (no candidate can change that: it is a property of the trace), and at any
    // time only the segments of conversations still going on are between the two.  So segments share rows: a
    // segment takes a slot at its first reference -- marked SEG_FRESH in that reference, where the replay resets
    // the row before anything reads it -- and gives it back after its last one.  Slots are reused oldest-first.
    std::vector<int64_t> last_ref((size_t)nseg, -1);
    for (int64_t r = 0; r < N; ++r)
        for (int64_t j = t->seg_off[(size_t)r]; j < t->seg_off[(size_t)r + 1]; ++j) last_ref[(size_t)t->seg[(size_t)j].id] = r;
    std::vector<int32_t> slot_of((size_t)nseg, -1);
    std::vector<int32_t> free_slots;       // a queue: taken from `head`, given back at the end
    size_t head = 0;
    int32_t n_slots = 0;
    std::vector<int32_t> seg_at;           // segments of the request in hand, by place in its path
    for (int64_t r = 0; r < N; ++r) {
        const int64_t j0 = t->seg_off[(size_t)r], j1 = t->seg_off[(size_t)r + 1];
        seg_at.clear();
        for (int64_t j = j0; j < j1; ++j) {
            gorgo::SegRef& ref = t->seg[(size_t)j];
            const size_t sg = (size_t)ref.id;
            seg_at.push_back(ref.id);
            if (slot_of[sg] < 0) {
                slot_of[sg] = head < free_slots.size() ? free_slots[head++] : n_slots++;
                ref.end |= gorgo::SEG_FRESH;
            }
            ref.id = slot_of[sg];
        }
        // (given back only now: a slot is not handed on within the request that still uses it)
        for (int64_t j = j0; j < j1; ++j) {
            const int32_t slot = t->seg[(size_t)j].id;
            if (last_ref[(size_t)seg_at[(size_t)(j - j0)]] == r) free_slots.push_back(slot);
        }
    }
    t->n_slots = n_slots;
    return GORGO_OK;
}

int check_and_finish(gorgo_trace* t, const int64_t* hash_ids, int32_t block_tokens) {
    if (block_tokens < 1) return fail(GORGO_ERR_INVALID_ARG, "block_tokens must be >= 1");
    const int64_t N = t->N;
    if (N >= 0x7FFFFFFF) return fail(GORGO_ERR_INVALID_ARG, "too many requests (limit 2^31-2)");
    if (t->blk_off[0] != 0) return fail(GORGO_ERR_INVALID_ARG, "blk_off[0] must be 0");
    for (int64_t r = 0; r < N; ++r) {
        if (r > 0 && t->ts[r] < t->ts[r - 1])
            return fail(GORGO_ERR_UNSORTED, "timestamps decrease at request " + std::to_string(r));
        if (t->ts[r] < 0) return fail(GORGO_ERR_INVALID_ARG, "negative timestamp at request " + std::to_string(r));
        if (t->ts[r] > (int64_t)1 << 53) return fail(GORGO_ERR_INVALID_ARG, "timestamp above 2^53 ms");
        if (t->in_len[r] < 0 || t->out_len[r] < 0)
            return fail(GORGO_ERR_INVALID_ARG, "negative token count at request " + std::to_string(r));
        const int64_t n = t->blk_off[r + 1] - t->blk_off[r];
        if (n < 0) return fail(GORGO_ERR_INVALID_ARG, "blk_off decreases at request " + std::to_string(r));
        if (n > 65535) return fail(GORGO_ERR_INVALID_ARG, "more than 65535 blocks in request " + std::to_string(r));
    }
    // the load signal (sum of input tokens in flight) is carried in fp64 and must stay an exact integer
    int64_t total_tokens = 0;
    for (int64_t r = 0; r < N; ++r) {
        total_tokens += t->in_len[r];
        if (total_tokens > ((int64_t)1 << 53)) return fail(GORGO_ERR_INVALID_ARG, "input tokens sum above 2^53");
    }
    t->block_tokens = block_tokens;
    // session-affinity policy (Sec. 4 "Baseline policies"): hash of the request's first block, here the high word
    // of the output that a SplitMix64 generator (Steele, Lea, Flood, OOPSLA'14) in state `id` gives next
    t->first_hash.assign((size_t)N, 0u);
    for (int64_t r = 0; r < N; ++r)
        if (t->blk_off[r + 1] > t->blk_off[r]) {
            uint64_t z = (uint64_t)hash_ids[t->blk_off[r]] + 0x9E3779B97F4A7C15ull;
            z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
            z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
            t->first_hash[(size_t)r] = (uint32_t)((z ^ (z >> 31)) >> 32);
        }
    return preprocess(t, hash_ids);
}

// ---- minimal JSON scanner (enough for flat objects with numbers, strings and arrays of numbers)
struct Cur {
    const char* p;
    const char* e;
    void ws() { while (p < e && (*p == ' ' || *p == '\t' || *p == '\r')) ++p; }
};

bool parse_int(Cur& c, int64_t* out) {
    c.ws();
    const char* s = c.p;
    bool neg = false;
    if (c.p < c.e && (*c.p == '-' || *c.p == '+')) { neg = *c.p == '-'; ++c.p; }
    if (c.p >= c.e || *c.p < '0' || *c.p > '9') { c.p = s; return false; }
    uint64_t v = 0;
    while (c.p < c.e && *c.p >= '0' && *c.p <= '9') {
        if (v > (std::numeric_limits<uint64_t>::max() - 9) / 10) return false;
        v = v * 10 + (uint64_t)(*c.p - '0');
        ++c.p;
    }
    // accept an integral float such as 12.0 or 1e3 only if it has no fractional/exponent part
    if (c.p < c.e && (*c.p == '.' || *c.p == 'e' || *c.p == 'E')) {
        char* endp = nullptr;
        std::string tmp(s, (size_t)std::min<ptrdiff_t>(c.e - s, 64));
        double d = std::strtod(tmp.c_str(), &endp);
        if (endp == tmp.c_str() || d != (double)(int64_t)d) return false;
        c.p = s + (endp - tmp.c_str());
        *out = (int64_t)d;
        return true;
    }
    if (!neg && v > (uint64_t)std::numeric_limits<int64_t>::max()) return false;
    *out = neg ? -(int64_t)v : (int64_t)v;
    return true;
}

bool skip_string(Cur& c) {
    if (c.p >= c.e || *c.p != '"') return false;
    ++c.p;
    while (c.p < c.e && *c.p != '"') {
        if (*c.p == '\\') ++c.p;
        ++c.p;
    }
    if (c.p >= c.e) return false;
    ++c.p;
    return true;
}

bool skip_value(Cur& c, int depth = 0) {
    c.ws();
    if (c.p >= c.e || depth > 32) return false;
    if (*c.p == '"') return skip_string(c);
    if (*c.p == '{' || *c.p == '[') {
        const char close = *c.p == '{' ? '}' : ']';
        const bool obj = *c.p == '{';
        ++c.p;
        c.ws();
        if (c.p < c.e && *c.p == close) { ++c.p; return true; }
        for (;;) {
            if (obj) {
                c.ws();
                if (!skip_string(c)) return false;
                c.ws();
                if (c.p >= c.e || *c.p != ':') return false;
                ++c.p;
            }
            if (!skip_value(c, depth + 1)) return false;
            c.ws();
            if (c.p < c.e && *c.p == ',') { ++c.p; continue; }
            if (c.p < c.e && *c.p == close) { ++c.p; return true; }
            return false;
        }
    }
    // number / true / false / null
    const char* s = c.p;
    while (c.p < c.e && *c.p != ',' && *c.p != '}' && *c.p != ']' && *c.p != ' ' && *c.p != '\t') ++c.p;
    return c.p > s;
}

// Parses one record.  Returns false on malformed input.
bool parse_line(const char* b, const char* e, int64_t* ts, int64_t* il, int64_t* ol, std::vector<int64_t>* ids,
                unsigned* have) {
    Cur c{b, e};
    c.ws();
    if (c.p >= c.e || *c.p != '{') return false;
    ++c.p;
    *have = 0;
    c.ws();
    if (c.p < c.e && *c.p == '}') return true;
    for (;;) {
        c.ws();
        const char* ks = c.p;
        if (!skip_string(c)) return false;
        std::string key(ks + 1, c.p - 1);
        c.ws();
        if (c.p >= c.e || *c.p != ':') return false;
        ++c.p;
        if (key == "timestamp") { if (!parse_int(c, ts)) return false; *have |= 1; }
        else if (key == "input_length") { if (!parse_int(c, il)) return false; *have |= 2; }
        else if (key == "output_length") { if (!parse_int(c, ol)) return false; *have |= 4; }
        else if (key == "hash_ids") {
            c.ws();
            if (c.p >= c.e || *c.p != '[') return false;
            ++c.p;
            c.ws();
            if (c.p < c.e && *c.p == ']') { ++c.p; }
            else {
                for (;;) {
                    int64_t v;
                    if (!parse_int(c, &v)) return false;
                    ids->push_back(v);
                    c.ws();
                    if (c.p < c.e && *c.p == ',') { ++c.p; continue; }
                    if (c.p < c.e && *c.p == ']') { ++c.p; break; }
                    return false;
                }
            }
            *have |= 8;
        } else if (!skip_value(c)) return false;
        c.ws();
        if (c.p < c.e && *c.p == ',') { ++c.p; continue; }
        if (c.p < c.e && *c.p == '}') { ++c.p; break; }
        return false;
    }
    c.ws();
    return c.p == c.e;
}

}  // namespace
}  // namespace gorgo

using namespace gorgo;

extern "C" {

const char* gorgo_last_error(void) { return g_err.c_str(); }

int gorgo_load_trace_arrays(int64_t N, const int64_t* ts_ms, const int32_t* in_len, const int32_t* out_len,
                            const int64_t* blk_off, const int64_t* hash_ids, int32_t block_tokens,
                            gorgo_trace** out) {
    clear_error();
    if (!out) return fail(GORGO_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (N < 0) return fail(GORGO_ERR_INVALID_ARG, "N is negative");
    if (!blk_off) return fail(GORGO_ERR_INVALID_ARG, "blk_off is NULL");
    if (N > 0 && (!ts_ms || !in_len || !out_len)) return fail(GORGO_ERR_INVALID_ARG, "a request array is NULL");
    if (N >= 0x7FFFFFFF) return fail(GORGO_ERR_INVALID_ARG, "too many requests (limit 2^31-2)");
    if (N > 0 && blk_off[N] > 0 && !hash_ids) return fail(GORGO_ERR_INVALID_ARG, "hash_ids is NULL");
    gorgo_trace* t = new (std::nothrow) gorgo_trace();
    if (!t) return fail(GORGO_ERR_OOM, "out of host memory");
    try {
        t->N = N;
        t->ts.assign(ts_ms, ts_ms + N);
        t->in_len.assign(in_len, in_len + N);
        t->out_len.assign(out_len, out_len + N);
        t->blk_off.assign(blk_off, blk_off + N + 1);
        int rc = check_and_finish(t, hash_ids, block_tokens);
        if (rc != GORGO_OK) { delete t; return rc; }
    } catch (const std::bad_alloc&) {
        delete t;
        return fail(GORGO_ERR_OOM, "out of host memory");
    }
    *out = t;
    return GORGO_OK;
}

int gorgo_load_trace(const char* jsonl_path, int32_t block_tokens, gorgo_trace** out) {
    clear_error();
    if (!out) return fail(GORGO_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!jsonl_path) return fail(GORGO_ERR_INVALID_ARG, "path is NULL");
    FILE* f = std::fopen(jsonl_path, "rb");
    if (!f) return fail(GORGO_ERR_IO, std::string("cannot open ") + jsonl_path + ": " + std::strerror(errno));
    std::vector<int64_t> ts, off, ids;
    std::vector<int32_t> il, ol;
    off.push_back(0);
    std::string line;
    char buf[1 << 16];
    int64_t lineno = 0;
    int rc = GORGO_OK;
    bool eof = false;
    try {
        while (!eof && rc == GORGO_OK) {
            line.clear();
            for (;;) {   // read one whole line of any length
                if (!std::fgets(buf, sizeof buf, f)) { eof = true; break; }
                size_t n = std::strlen(buf);
                if (n && buf[n - 1] == '\n') { line.append(buf, n - 1); break; }
                line.append(buf, n);
            }
            if (std::ferror(f)) { rc = fail(GORGO_ERR_IO, std::string("read error on ") + jsonl_path); break; }
            ++lineno;
            size_t a = line.find_first_not_of(" \t\r");
            if (a == std::string::npos) continue;   // blank line
            int64_t t0 = 0, i0 = 0, o0 = 0;
            unsigned have = 0;
            size_t before = ids.size();
            if (!parse_line(line.data(), line.data() + line.size(), &t0, &i0, &o0, &ids, &have)) {
                rc = fail(GORGO_ERR_PARSE, "malformed record on line " + std::to_string(lineno));
                break;
            }
            if (have != 15u) {
                rc = fail(GORGO_ERR_PARSE, "line " + std::to_string(lineno) +
                                               ": needs timestamp, input_length, output_length and hash_ids");
                break;
            }
            if (i0 < 0 || i0 > 0x7FFFFFFF || o0 < 0 || o0 > 0x7FFFFFFF) {
                rc = fail(GORGO_ERR_PARSE, "line " + std::to_string(lineno) + ": token count out of range");
                break;
            }
            (void)before;
            ts.push_back(t0);
            il.push_back((int32_t)i0);
            ol.push_back((int32_t)o0);
            off.push_back((int64_t)ids.size());
        }
    } catch (const std::bad_alloc&) {
        rc = fail(GORGO_ERR_OOM, "out of host memory");
    }
    std::fclose(f);
    if (rc != GORGO_OK) return rc;
    return gorgo_load_trace_arrays((int64_t)ts.size(), ts.data(), il.data(), ol.data(), off.data(), ids.data(),
                                   block_tokens, out);
}

int gorgo_trace_info(const gorgo_trace* t, int64_t* N, int64_t* total_blocks, int32_t* max_blocks,
                     int64_t* unique_ids, int32_t* chain_consistent) {
    clear_error();
    if (!t) return fail(GORGO_ERR_INVALID_ARG, "trace is NULL");
    if (N) *N = t->N;
    if (total_blocks) *total_blocks = t->total_blocks;
    if (max_blocks) *max_blocks = t->max_blocks;
    if (unique_ids) *unique_ids = t->unique_ids;
    if (chain_consistent) *chain_consistent = t->chain_consistent ? 1 : 0;
    return GORGO_OK;
}

void gorgo_free_trace(gorgo_trace* t) {
    if (!t) return;
    release_device_trace(t);
    delete t;
}

}  // extern "C"
