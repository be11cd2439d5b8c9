"""Summarises the `kernels` view of a rocprofv3 result database (rocpd/sqlite): per-kernel count,
average/min/max/total duration, and the gaps between consecutive kernels.

  python -m paper_2411_03786_amd.prof_summary <output dir>/bench_results.db [rows]
"""
import sqlite3, sys, re
db=sqlite3.connect(sys.argv[1]); cur=db.cursor()
rows=cur.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) from kernels group by name order by 6 desc").fetchall()
tot=sum(r[5] for r in rows)
print(f"total kernel time {tot/1e6:.2f} ms")
for r in rows[:int(sys.argv[2]) if len(sys.argv)>2 else 30]:
    n=r[0].replace('ngg::','').replace('void ','')
    print(f"{n[:100]:100s} n={r[1]:6d} avg={r[2]/1e3:8.1f}us min={r[3]/1e3:7.1f} max={r[4]/1e3:8.1f} tot={r[5]/1e6:8.2f}ms {100*r[5]/tot:5.1f}%")
# timeline gaps for the last verify step: find last argmax_accept dispatch with k>0 ... simply report gaps stats between consecutive kernels on the busiest stream
rows=cur.execute("select start,end,name from kernels order by start").fetchall()
gaps=[rows[i+1][0]-rows[i][1] for i in range(len(rows)-1)]
import statistics
g=[x for x in gaps if 0<=x<50000]
print("gaps: n=%d median=%.2fus mean=%.2fus"%(len(g), statistics.median(g)/1e3, sum(g)/len(g)/1e3))
