"""Host-side emulation of the index arithmetic of the persistent 3x3 convolution kernel
(k_conv3x3_v4 in csrc/dnb_conv_f32_fast.hip): for every workgroup, tile, thread and staging slot it
recomputes the addresses the kernel forms -- global loads of the input rows, packed-weight loads,
LDS stores of the staged rows, LDS operand reads of the nine taps, the statistics scratch and the
output stores -- with the kernel's own constants (plane pitch 144, row pitch W + 4, 512 workgroups
dealt to 8 XCDs) and checks that each stays inside its buffer and that every tile is taken exactly
once.  An earlier version of the kernel overran the last staged row by one float; this is the
check that found it.  CPU only: nothing is launched."""
import pytest


def check(n, cin, cout, H, W, label, sample=None):
    HW=H*W; mtiles=(cout+15)//16; M16=mtiles*16; K16=(cin+15)//16*16; nch=K16//16
    assert (mtiles,nch) in ((1,3),(3,1)) and W in (8,16,32) and HW%64==0
    MT,NCH=mtiles,nch; ROWS=NCH*16; RW=W+4; TR=64//W; NR=TR+2; W4=W//4; CS=144
    assert NR*RW<=CS
    PER=NR*W4; TOTAL=ROWS*PER; U=(TOTAL+255)//256; BUF=ROWS*CS+4; SST0=2*BUF
    lds_floats=2*(NCH*16*144+4)+2*4*mtiles*16*3
    tpi=HW//64; total_tiles=tpi*n
    G=(total_tiles+7)//8*8 if total_tiles<512 else 512
    tpx=(total_tiles+7)>>3; wgx=G>>3
    in_elems=n*cin*HW; out_elems=n*cout*HW; w_elems=9*M16*K16
    wgs=range(G) if sample is None or G<=2*sample else list(range(sample))+list(range(G-sample,G))
    full=len(list(wgs))==G; done=set(); bad=0
    for b in wgs:
        xcd=b&7; slot=b>>3; t_lo=xcd*tpx; t_hi=min(total_tiles,t_lo+tpx); tile=t_lo+slot
        it=0
        while tile<t_hi:
            assert tile not in done; done.add(tile)
            img=tile//tpi; y0=(tile-img*tpi)*TR
            for tid in range(256):
                lane=tid&63; wave=tid>>6; j=lane&15; g=lane>>4
                for u in range(U):
                    idx=min(u*256+tid,TOTAL-1); sch=idx//PER; rem=idx-sch*PER; sry=rem//W4; sgo=4*(rem-sry*W4)
                    slo=sch*CS+sry*RW+4+sgo
                    y=min(max(y0-1+sry,0),H-1)
                    a=img*cin*HW+min(sch,cin-1)*HW+y*W+sgo
                    if not(0<=a and a+3<in_elems): bad+=1
                    if u*256+tid<TOTAL:
                        for boff in (0,BUF):
                            if not(0<=boff+slo and boff+slo+3<boff+BUF-4): bad+=1
                for t in range(9):
                    for a_ in range(MT):
                        for ci in range(NCH):
                            wa=((t*M16+a_*16+j)*K16+ci*16+4*g)
                            if not(0<=wa and wa+3<w_elems): bad+=1
                p=16*wave+j; base=g*CS+(p//W+1)*RW+4+(p%W)
                for boff in (0,BUF):
                    for ci in range(NCH):
                        for di in (-1,0,1):
                            for dj in (-1,0,1):
                                for ks in range(4):
                                    l=boff+base+(ci*16+4*ks)*CS+di*RW+dj
                                    if not(boff<=l<boff+BUF): bad+=1
                q=(tile-img*tpi)*64+p
                assert q<HW
                for a_ in range(MT):
                    for r in range(4):
                        m=a_*16+4*g+r
                        if m<cout:
                            o=img*cout*HW+q+m*HW
                            if not(0<=o<out_elems): bad+=1
                        sidx=SST0+(((1*4+wave)*(MT*16))+a_*16+4*g+r)*3
                        if not(sidx+2<lds_floats): bad+=1
            tile+=wgx; it+=1
    assert (not full) or done==set(range(total_tiles)), label
    return bad, lds_floats * 4


CASES = [
    (2, 48, 12, 8, 8, "fwd 8x8", None),
    (2, 12, 48, 8, 8, "dgrad 8x8", None),
    (2, 48, 12, 32, 32, "fwd 32x32", None),
    (3, 12, 48, 16, 16, "dgrad 16x16 n3", None),
    (64, 48, 12, 32, 32, "fwd, first block of DenseNet-BC-100 at batch 64", 6),
    (64, 12, 48, 32, 32, "dgrad, first block", 6),
    (64, 48, 12, 16, 16, "fwd, second block", 6),
    (64, 12, 48, 16, 16, "dgrad, second block", 6),
    (64, 48, 12, 8, 8, "fwd, third block", None),
    (64, 12, 48, 8, 8, "dgrad, third block", None),
    (4, 40, 12, 8, 8, "fwd, 40 input channels (channel tail)", None),
    (2, 12, 40, 8, 16, "dgrad, 40 output channels, 8x16 image", None),
]


@pytest.mark.parametrize("n,cin,cout,H,W,label,sample", CASES, ids=[c[5] for c in CASES])
def test_every_access_of_the_persistent_3x3_kernel_is_in_bounds(n, cin, cout, H, W, label, sample):
    bad, lds_bytes = check(n, cin, cout, H, W, label, sample)
    assert bad == 0
    assert lds_bytes <= 64 * 1024
