// host-only sanitizer run over build_layout / build_work_tiles with random layouts
#include "layout.hpp"
#include <cstdio>
#include <random>
using namespace ffsnap;
int main(){
  std::mt19937_64 rng(1);
  static char arena[1<<20];
  for(int it=0; it<3000; it++){
    int n = 1 + rng()%40;
    std::vector<ff_segment> segs;
    uint64_t chunk = 1024ull << (rng()%14);
    bool groups = rng()%2;
    if(groups){
      int np = 1 + rng()%8;
      for(int p=0;p<np;p++){ uint64_t ne = rng()%3==0 ? 1 + rng()%5 : 1 + rng()%200000;
        uint32_t half = (rng()%2)? FF_BF16: FF_F16; if(rng()%5) half=FF_BF16;
        segs.push_back({arena+2, 2*ne, half, FF_KIND_W16, (uint32_t)p, 0});
        segs.push_back({arena+4, 4*ne, FF_F32, FF_KIND_MASTER, (uint32_t)p, 0});
        segs.push_back({arena+8, 4*ne, FF_F32, FF_KIND_M, (uint32_t)p, 0});
        segs.push_back({arena+12, 4*ne, FF_F32, FF_KIND_V, (uint32_t)p, 0});
        if(rng()%3==0) segs.push_back({arena+2, 2*(rng()%3000), FF_BF16, FF_KIND_RAW, 0, 0});
      }
    } else {
      for(int i=0;i<n;i++){ uint32_t dt = 1 + rng()%3; uint64_t es = dt==FF_F32?4:2; segs.push_back({arena+es, es*(rng()%100000), dt, FF_KIND_RAW, 0, 0}); }
    }
    Layout L; unsigned tl = rng()%3==0 ? 10 + rng()%12 : 0;
    int rc = build_layout(segs.data(), segs.size(), chunk, tl, L);
    if(rc!=FF_OK) continue;
    // invariants
    if(L.n_tiles != L.n_chunks * L.tiles_per_chunk || L.tile_first_seg.size()!=L.n_tiles){ printf("tiling mismatch\n"); return 1; }
    for(uint64_t t=0;t<L.n_tiles;t++){ uint64_t s=t*L.tile_bytes; uint32_t f=L.tile_first_seg[t]; if(f>=L.segs.size()){printf("first seg range\n");return 1;}
      if(s<L.payload && !(L.segs[f].off<=s && s<L.segs[f].off+L.segs[f].nbytes)){printf("first seg wrong\n");return 1;} }
    if(L.tile_base.size()!=L.n_tiles){ printf("tile_base size\n"); return 1; }
    for(uint64_t t=0;t<L.n_tiles;t++){ uint64_t s=t*L.tile_bytes, e=s+L.tile_bytes; uint64_t want=0;
      for(auto& g: L.segs) if(g.off<=s && e<=g.off+g.nbytes) want=g.ptr+(s-g.off);
      if(L.tile_base[t]!=want){ printf("tile_base wrong\n"); return 1; } }
    if(L.adam_ok && !L.params.empty()){
      std::vector<WorkTile> w; build_work_tiles(L,w);
      // every payload byte covered exactly once by the tiles' streams
      uint64_t covered=0;
      for(auto&t:w){ if(t.kind==kWorkParam) covered += 14ull*t.n; else covered += t.n; for(int x=0;x<7;x++) if(t.shift[x] && t.chunk[x]>=L.n_chunks){printf("chunk range\n");return 1;} }
      if(covered!=L.payload){ printf("coverage %llu vs %llu\n",(unsigned long long)covered,(unsigned long long)L.payload); return 1; }
    }
  }
  printf("ok\n"); return 0;
}
