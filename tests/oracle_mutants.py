"""Mutation check of the oracle pins (run by hand: `python tests/oracle_mutants.py`,
about two minutes, CPU only).  Each entry plants one plausible mistake in a copy
of oracle/gnnd_oracle.c under /tmp and runs tests/test_oracle_pins.py against
it; every mutant has to fail.  Nothing here touches the GPU or the product."""
import subprocess, shutil, os, sys
muts = [
 ("hash drops c", "h = og_mix64(h + (uint64_t)c);", "h = og_mix64(h);"),
 ("bounded uses low bits", "return (uint32_t)(((h >> 32) * (uint64_t)n) >> 32);", "return (uint32_t)((h & 0xffffffffu) % n);"),
 ("l2 unfused", "acc = fmaf(diff, diff, acc);", "acc = acc + diff * diff;"),
 ("dot sign", "return (double)(1.0f - dot);", "return (double)(1.0f + dot);"),
 ("u8 abs not square", "acc += diff * diff;", "acc += diff < 0 ? -diff : diff;"),
 ("closer ignores id", "return d1 < d2 || (d1 == d2 && id1 < id2);", "return d1 < d2;"),
 ("bf includes self", "if (c == s) continue;", "if (c == -5) continue;"),
 ("init allows self", "(uint32_t)n, 0, (int32_t)s, draw);", "(uint32_t)n, 0, -1, draw);"),
 ("sample new cap off by one", "if (a < p) {", "if (a <= p) {"),
 ("sample flag not cleared", "          isnew[s * k + j] = 0;\n", ""),
 ("rev key ignores iter", "og_hash(seed, tag, (uint32_t)v, (uint32_t)s, iter)", "og_hash(seed, tag, (uint32_t)v, (uint32_t)s, 0)"),
 ("rev room ignores forward", "int room = cap2p - m;", "int room = cap2p;"),
 ("rev no dedupe", "if (j == 0 || list[j] != list[j - 1]) out[v * cap2p + u++] = list[j];", "out[v * cap2p + u++] = list[j];"),
 ("rev sort by s not key", "if (a->key != b->key) return a->key < b->key ? -1 : 1;", ""),
 ("pair map floor", "ceil(sqrt(2.0 * (double)t + 2.25) - 0.5)", "floor(sqrt(2.0 * (double)t + 2.25) - 0.5)"),
 ("join same-id not skipped", "int ok = N[a] != O[b];", "int ok = 1;"),
 ("join merge filter dropped", "if (ok && split >= 0) ok = ((N[a] < split) != (O[b] < split));", ""),
 ("join nn uses max instead of min", "if (best < 0 || closer(dist, N[c], bd, N[best])) {\n            best = c;", "if (best < 0 || !closer(dist, N[c], bd, N[best])) {\n            best = c;"),
 ("join old->new proposal dest swapped", "qu[m] = O[b];\n        qv[m] = N[best];", "qu[m] = N[best];\n        qv[m] = O[b];"),
 ("update keeps k+1th", "for (int64_t e = 0; e < m && w < k; ++e) {\n      int dup = 0;\n      for (int j = 0; j < w && !dup; ++j) dup = (ids[u * k + j] == pool[e].id);", "for (int64_t e = 1; e < m && w < k; ++e) {\n      int dup = 0;\n      for (int j = 0; j < w && !dup; ++j) dup = (ids[u * k + j] == pool[e].id);"),
 ("update no dedupe", "for (int j = 0; j < w && !dup; ++j) dup = (ids[u * k + j] == pool[e].id);\n      if (dup) continue;\n      ids[u * k + w] = pool[e].id;\n      dist[u * k + w] = pool[e].d;\n      isnew[u * k + w] = pool[e].isnew;", "ids[u * k + w] = pool[e].id;\n      dist[u * k + w] = pool[e].d;\n      isnew[u * k + w] = pool[e].isnew;"),
 ("update new flag lost", "pool[m].isnew = 1;\n      pool[m].fresh = 1;", "pool[m].isnew = 0;\n      pool[m].fresh = 1;"),
 ("insert_one accepts dup", "if (ids[j] == v) return 0;", "if (ids[j] == -7) return 0;"),
 ("merge keep floor", "const int keep = (k + 1) / 2, fill = k / 2;\n  const int64_t n = n1 + n2;", "const int keep = k / 2, fill = (k + 1) / 2;\n  const int64_t n = n1 + n2;"),
 ("merge fill from own set", "draw_distinct(seed, OG_TAG_MERGE, (uint32_t)s, fill, (uint32_t)(first ? n2 : n1),\n                  first ? (int32_t)n1 : 0, -1, draw);", "draw_distinct(seed, OG_TAG_MERGE, (uint32_t)s, fill, (uint32_t)(first ? n1 : n2),\n                  first ? 0 : (int32_t)n1, -1, draw);"),
 ("merge fill flagged old", "row[keep + j].isnew = 1;", "row[keep + j].isnew = 0;"),
 ("frozen sampled", "if (v < 0 || v >= n) continue;", "if (v < 0) continue;"),
 ("to_global wrong base", "return (int32_t)(base2 + i - n1);", "return (int32_t)(base1 + i);"),
 ("all-pairs one way only", "          qu[m] = N[a]; qv[m] = N[b]; qd[m] = dist; ++m;\n          qu[m] = N[b]; qv[m] = N[a]; qd[m] = dist; ++m;", "          qu[m] = N[a]; qv[m] = N[b]; qd[m] = dist; ++m;"),
 ("all-pairs same id not skipped", "        if (N[a] == O[b]) continue;\n        if (split >= 0", "        if (split >= 0"),
 ("all-pairs old x old evaluated", "        qu[m] = N[a]; qv[m] = O[b]; qd[m] = dist; ++m;\n        qu[m] = O[b]; qv[m] = N[a]; qd[m] = dist; ++m;", "        qu[m] = N[a]; qv[m] = O[b]; qd[m] = dist; ++m;\n        qu[m] = O[b]; qv[m] = O[b > 0 ? b - 1 : 0]; qd[m] = dist; ++m;"),
 ("update rows stride", "return og_update_rows(n, k, 6 * p, ids, dist, isnew, pu, pv, pd, pcnt);", "return og_update_rows(n, k, 6 * p + 1, ids, dist, isnew, pu, pv, pd, pcnt);"),
 ("chi2 divides by the difference", "      acc = acc + sq / sum;", "      acc = acc + sq / (diff != 0.0f ? diff : 1.0f);"),
 ("chi2 fused", "      const float sq = diff * diff;\n      acc = acc + sq / sum;", "      acc = fmaf(diff, diff / sum, acc);"),
 ("chi2 counts empty dimensions", "    if (sum > 0.0f) {\n      const float sq = diff * diff;", "    if (sum >= 0.0f) {\n      const float sq = diff * diff;"),
 ("cosine without the root", "  const float den = sqrtf(na * nb);", "  const float den = na * nb;"),
 ("cosine norm of the wrong vector", "  const float nb = dot_f32(b, b, d);", "  const float nb = dot_f32(a, a, d);"),
 ("cosine zero vector at distance 0", "  return den > 0.0f ? 1.0f - dot / den : 1.0f;", "  return den > 0.0f ? 1.0f - dot / den : 0.0f;"),
 ("cosine two roots", "  const float den = sqrtf(na * nb);", "  const float den = sqrtf(na) * sqrtf(nb);"),
 ("merge final without the set-aside half", "    for (int j = 0; j < fill; ++j) {\n      pool[m].id = aside_ids[s * fill + j];", "    for (int j = 0; j < 0; ++j) {\n      pool[m].id = aside_ids[s * fill + j];"),
 ("merge sets aside one entry twice", "aside_ids[s * fill + j] = og_to_internal(sid[keep + j], n1, base1, n2, base2);\n      aside_dist[s * fill + j] = sdist[keep + j];", "aside_ids[s * fill + j] = og_to_internal(sid[keep + (j ? j - 1 : 0)], n1, base1, n2, base2);\n      aside_dist[s * fill + j] = sdist[keep + (j ? j - 1 : 0)];"),
 ("merge fill distance to the wrong node", "row[keep + j].d = og_distance(metric, d, vec, s, draw[j]);", "row[keep + j].d = og_distance(metric, d, vec, s > 0 ? s - 1 : s, draw[j]);"),
 ("segment capacity ignored", "      if (held[pool[e].id % classes] >= k / classes) continue;  /* its segment is full */\n", ""),
 ("segment chosen by position not id", "      if (held[pool[e].id % classes] >= k / classes) continue;  /* its segment is full */\n      held[pool[e].id % classes]++;", "      if (held[w % classes] >= k / classes) continue;\n      held[w % classes]++;"),
 ("segmented init ignores the class", "        const int32_t id = draw[j] * m + r;", "        const int32_t id = draw[j] * m;"),
 ("segmented init may draw the node itself", "      const int32_t own = (s % m == r) ? (int32_t)(s / m) : -1;  /* s as a member number */", "      const int32_t own = -1;"),
 ("segmented init reuses slot numbers", "draw_distinct_from(seed, OG_TAG_INIT, (uint32_t)s, 32 * r, 32, members, 0, own, draw);", "draw_distinct_from(seed, OG_TAG_INIT, (uint32_t)s, 0, 32, members, 0, own, draw);"),
 ("classic inserts one side only", "        ins += (uint64_t)og_insert_one(k, ids + (int64_t)N[b] * k, dist + (int64_t)N[b] * k,\n                                       isnew + (int64_t)N[b] * k, N[a], dd);\n", ""),
]
root=os.path.dirname(os.path.dirname(os.path.abspath(__file__))); tmp="/tmp/gnnd_oracle_mutants"
src=open(root+"/oracle/gnnd_oracle.c").read()
survived=[]
for name, old, new in muts:
    if src.count(old)!=1:
        print("SKIP (pattern count %d): %s"%(src.count(old),name)); continue
    shutil.rmtree(tmp, ignore_errors=True)
    os.makedirs(tmp+"/oracle"); os.makedirs(tmp+"/tests/golden")
    for f in ("oracle/__init__.py","oracle/gnnd_oracle.py","workloads.py","tests/conftest.py","tests/test_oracle_pins.py","tests/golden/splitmix64_seed0.txt"):
        shutil.copy(root+"/"+f, tmp+"/"+f)
    open(tmp+"/oracle/gnnd_oracle.c","w").write(src.replace(old,new))
    r=subprocess.run([sys.executable,"-m","pytest","tests/test_oracle_pins.py","-x","-q","-p","no:cacheprovider"],cwd=tmp,capture_output=True,text=True,timeout=600)
    ok = r.returncode==0
    print(("SURVIVED  " if ok else "killed    ")+name, flush=True)
    if ok: survived.append(name)
print("survivors:", survived)
sys.exit(1 if survived else 0)
