"""Hardware probes: `python -m paper_2305_10727_amd.probes [--out PREFIX]` compiles probes/hw_probes.hip with hipcc (the GPU
box carries the same ROCm image), runs it on the current GPU and writes PREFIX.txt / PREFIX.json: measured matrix
instruction rates, stream bandwidth, LDS and global->LDS rates per CU, and the shader clock under load.  These are the
measured denominators quoted beside the nominal peaks; profiles/hardware_probes.* is a committed run of this program."""
