#include "layout.hpp"

#include <algorithm>
#include <map>

#include "gf2.h"

namespace ffsnap {

static bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

int build_layout(const ff_segment* segs, uint64_t n_segs, uint64_t chunk_bytes, unsigned tile_log2,
                 Layout& L)
{
    if (n_segs && !segs) return FF_ERR_NULL;
    if (!is_pow2(chunk_bytes) || chunk_bytes < FF_MIN_CHUNK_BYTES || chunk_bytes > FF_MAX_CHUNK_BYTES)
        return FF_ERR_INVALID;
    if (n_segs >= 0xFFFFFFFFull) return FF_ERR_INVALID;

    L = Layout();
    L.chunk_bytes = chunk_bytes;
    uint64_t off = 0;
    for (uint64_t i = 0; i < n_segs; i++) {
        const ff_segment& s = segs[i];
        if (s.dtype != FF_BF16 && s.dtype != FF_F32 && s.dtype != FF_F16) return FF_ERR_INVALID;
        if (s.kind > FF_KIND_V || s.reserved != 0) return FF_ERR_INVALID;
        const uint64_t es = (s.dtype == FF_F32) ? 4 : 2;
        if (s.nbytes % es) return FF_ERR_INVALID;
        if (s.nbytes == 0) continue;  // empty segments take no place in the stream
        if (!s.ptr) return FF_ERR_NULL;
        if (reinterpret_cast<uint64_t>(s.ptr) % es) return FF_ERR_INVALID;
        if (off + s.nbytes < off) return FF_ERR_INVALID;
        L.segs.push_back(Seg{reinterpret_cast<uint64_t>(s.ptr), off, s.nbytes, s.dtype, s.kind,
                             s.param_id});
        off += s.nbytes;
    }
    if (off == 0) return FF_ERR_EMPTY;
    L.payload = off;
    L.n_chunks = (off + chunk_bytes - 1) / chunk_bytes;
    L.buffer_bytes = L.n_chunks * chunk_bytes;

    // layout id: CRC32C over (chunk_bytes, nbytes...) as little-endian uint64
    {
        std::vector<uint64_t> key;
        key.reserve(L.segs.size() + 1);
        key.push_back(chunk_bytes);
        for (const Seg& s : L.segs) key.push_back(s.nbytes);
        L.layout_id = crc32c_host(key.data(), key.size() * sizeof(uint64_t));
    }

    // parameter groups
    {
        std::map<uint32_t, Param> groups;
        bool ok = true;
        for (size_t i = 0; i < L.segs.size(); i++) {
            const Seg& s = L.segs[i];
            if (s.kind == FF_KIND_RAW) continue;
            auto it = groups.find(s.param_id);
            if (it == groups.end())
                it = groups.emplace(s.param_id, Param{s.param_id, {-1, -1, -1, -1}, 0}).first;
            int32_t& slot = it->second.seg[s.kind - 1];
            if (slot >= 0) ok = false;  // the same role twice
            slot = static_cast<int32_t>(i);
            // working weights are 16-bit, of one format throughout the plan; the rest is fp32
            if (s.kind == FF_KIND_W16) {
                if (s.dtype == FF_F32) ok = false;
                if (L.half_dtype == 0) L.half_dtype = s.dtype;
                if (s.dtype != L.half_dtype) ok = false;
            } else if (s.dtype != FF_F32) {
                ok = false;
            }
        }
        for (auto& kv : groups) {
            Param& p = kv.second;
            bool complete = p.seg[0] >= 0 && p.seg[1] >= 0 && p.seg[2] >= 0 && p.seg[3] >= 0;
            if (!complete) { ok = false; continue; }
            p.numel = L.segs[p.seg[1]].nbytes / 4;
            if (L.segs[p.seg[0]].nbytes != 2 * p.numel || L.segs[p.seg[2]].nbytes != 4 * p.numel ||
                L.segs[p.seg[3]].nbytes != 4 * p.numel)
                ok = false;
            L.params.push_back(p);
        }
        L.adam_ok = ok;
        if (!ok) L.params.clear();
    }

    // tiling
    uint64_t tile = kDefaultTileBytes;
    if (tile_log2) tile = 1ull << std::min<unsigned>(std::max<unsigned>(tile_log2, 10), 30);
    tile = std::min(tile, chunk_bytes);
    L.tile_bytes = tile;
    L.tiles_per_chunk = static_cast<uint32_t>(chunk_bytes / tile);
    L.n_tiles = L.buffer_bytes / tile;
    L.tile_first_seg.resize(L.n_tiles);
    size_t si = 0;
    for (uint64_t k = 0; k < L.n_tiles; k++) {
        const uint64_t s = k * tile;
        while (si + 1 < L.segs.size() && L.segs[si].off + L.segs[si].nbytes <= s) si++;
        L.tile_first_seg[k] = static_cast<uint32_t>(si);
    }
    L.tile_base.assign(L.n_tiles, 0);
    for (uint64_t k = 0; k < L.n_tiles; k++) {
        const uint64_t s = k * tile;
        const Seg& g = L.segs[L.tile_first_seg[k]];
        if (g.off <= s && s + tile <= g.off + g.nbytes) L.tile_base[k] = g.ptr + (s - g.off);
    }
    return FF_OK;
}

namespace {

uint32_t shift_to_chunk_end(uint64_t piece_end, uint64_t chunk_bytes)
{
    const uint64_t chunk_end = (piece_end + chunk_bytes - 1) / chunk_bytes * chunk_bytes;
    return gf2_xpow(8 * (chunk_end - piece_end));
}

}  // namespace

void build_work_tiles(const Layout& L, std::vector<WorkTile>& out)
{
    out.clear();
    const uint64_t C = L.chunk_bytes;
    std::vector<bool> in_group(L.segs.size(), false);
    for (size_t pi = 0; pi < L.params.size(); pi++) {
        const Param& p = L.params[pi];
        const uint64_t size[4] = {2, 4, 4, 4};
        uint64_t off[4], ptr[4];
        for (int x = 0; x < 4; x++) {
            off[x] = L.segs[p.seg[x]].off;
            ptr[x] = L.segs[p.seg[x]].ptr;
            in_group[p.seg[x]] = true;
        }
        // cut points: (element, streams whose element is split there)
        std::map<uint64_t, uint32_t> cuts;
        cuts[0] = 0;
        for (int x = 0; x < 4; x++) {
            const uint64_t a = off[x], b = off[x] + size[x] * p.numel;
            for (uint64_t B = (a / C + 1) * C; B < b; B += C) {
                const uint64_t e = (B - a) / size[x];
                uint32_t& m = cuts[e];
                if ((B - a) % size[x]) m |= 1u << x;
            }
        }
        for (auto it = cuts.begin(); it != cuts.end(); ++it) {
            auto nx = std::next(it);
            const uint64_t end = (nx == cuts.end()) ? p.numel : nx->first;
            for (uint64_t e0 = it->first; e0 < end; e0 += kParamTileElems) {
                WorkTile t{};
                t.kind = kWorkParam;
                t.grad_index = static_cast<uint32_t>(pi);
                t.e0 = e0;
                t.n = static_cast<uint32_t>(std::min<uint64_t>(kParamTileElems, end - e0));
                t.head_split = (e0 == it->first) ? it->second : 0;
                for (int x = 0; x < 4; x++) {
                    t.ptr[x] = ptr[x] + size[x] * e0;
                    t.soff[x] = off[x] + size[x] * e0;
                    uint64_t begin = t.soff[x];
                    const uint64_t stop = t.soff[x] + size[x] * t.n;
                    if (t.head_split & (1u << x)) {
                        t.chunk[3 + x] = static_cast<uint32_t>(begin / C);
                        t.shift[3 + x] = kOne;  // the two head bytes end their chunk
                        begin += 2;
                    }
                    t.chunk[x] = static_cast<uint32_t>(begin / C);
                    t.shift[x] = shift_to_chunk_end(stop, C);
                }
                out.push_back(t);
            }
        }
    }
    for (size_t i = 0; i < L.segs.size(); i++) {
        if (in_group[i]) continue;
        const Seg& s = L.segs[i];
        uint64_t pos = 0;
        while (pos < s.nbytes) {
            const uint64_t abs = s.off + pos;
            uint64_t len = std::min<uint64_t>(kRawTileBytes, s.nbytes - pos);
            len = std::min<uint64_t>(len, (abs / C + 1) * C - abs);
            WorkTile t{};
            t.kind = kWorkRaw;
            t.n = static_cast<uint32_t>(len);
            t.ptr[0] = s.ptr + pos;
            t.soff[0] = abs;
            t.chunk[0] = static_cast<uint32_t>(abs / C);
            t.shift[0] = shift_to_chunk_end(abs + len, C);
            out.push_back(t);
            pos += len;
        }
    }
}

}  // namespace ffsnap
